// Host-only driver for the library's planner and argument checks, built with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host side (tests/test_host_sanitized.py compiles csrc/ckv_host.hip
// together with this file; the kernel launchers resolve from libckv.so and are never reached: every
// call made here returns before any launch).  Reads one command per line from stdin and prints one
// result line per command, which the test compares with what the regular library returns for the
// same arguments.
#include <stdio.h>
#include <string.h>

#include <iostream>
#include <sstream>
#include <string>
#include <vector>

#include "ckv.h"

static ckv_params read_params(std::istringstream& in) {
  ckv_params p;
  memset(&p, 0, sizeof(p));
  in >> p.chunk >> p.retain_ratio >> p.n_rounds;
  for (int j = 0; j < CKV_MAX_ROUNDS; ++j) in >> p.r[j];
  in >> p.n_sink >> p.n_recent >> p.scope >> p.flags;
  return p;
}

static ckv_layout read_layout(std::istringstream& in) {
  ckv_layout l;
  memset(&l, 0, sizeof(l));
  in >> l.batch >> l.heads >> l.seq >> l.dim >> l.stride_b >> l.stride_h >> l.stride_s >> l.dtype >> l.deg_stride;
  return l;
}

static ckv_paged_layout read_paged(std::istringstream& in) {
  ckv_paged_layout pl;
  memset(&pl, 0, sizeof(pl));
  in >> pl.batch >> pl.heads >> pl.dim >> pl.dtype >> pl.block_size >> pl.max_blocks >> pl.n_blocks;
  return pl;
}

int main() {
  std::string line;
  void* fake = reinterpret_cast<void*>(4096);   // never dereferenced: the calls that take it fail validation first
  while (std::getline(std::cin, line)) {
    std::istringstream in(line);
    std::string cmd;
    if (!(in >> cmd)) continue;
    if (cmd == "plan") {
      ckv_layout l = read_layout(in);
      ckv_params p = read_params(in);
      ckv_plan_t plan;
      memset(&plan, 0, sizeof(plan));
      const int st = ckv_plan(&l, &p, &plan);
      printf("plan %d %d %d", st, plan.out_seq, plan.n_rounds);
      for (int j = 0; j <= CKV_MAX_ROUNDS; ++j) printf(" %d", plan.round_len[j]);
      for (int j = 0; j < CKV_MAX_ROUNDS; ++j) printf(" %.9g", plan.round_r[j]);
      printf(" %zu\n", plan.workspace_bytes);
    } else if (cmd == "anneal") {
      int seq, chunk, n_sink, n_recent, scope, budget;
      float r_init, delta, r_floor;
      in >> seq >> chunk >> n_sink >> n_recent >> scope >> budget >> r_init >> delta >> r_floor;
      ckv_params p;
      memset(&p, 0, sizeof(p));
      const int st = ckv_schedule_annealed(seq, chunk, n_sink, n_recent, scope, budget, r_init, delta, r_floor, &p);
      printf("anneal %d %d", st, p.n_rounds);
      for (int j = 0; j < CKV_MAX_ROUNDS; ++j) printf(" %.9g", p.r[j]);
      printf("\n");
    } else if (cmd == "pplan") {
      ckv_paged_layout pl = read_paged(in);
      int seq, n_lens;
      in >> seq >> n_lens;
      std::vector<int32_t> lens(n_lens);
      for (int i = 0; i < n_lens; ++i) in >> lens[i];
      ckv_params p = read_params(in);
      std::vector<int32_t> out(n_lens > 0 ? n_lens : 1, -1);
      int32_t n_freed = -1;
      size_t bytes = 0;
      const int st = ckv_paged_compress_plan(&pl, seq, n_lens > 0 ? lens.data() : nullptr, &p, out.data(), &n_freed, &bytes);
      printf("pplan %d %d %zu", st, n_freed, bytes);
      for (int32_t v : out) printf(" %d", v);
      printf("\n");
    } else if (cmd == "sizes") {
      int seq, chunk, n, old_seq, new_seq;
      float ratio;
      in >> seq >> chunk >> ratio >> n;
      ckv_paged_layout pl = read_paged(in);
      in >> old_seq >> new_seq;
      printf("sizes %d %d %d\n", ckv_n_sources(seq, chunk), ckv_budget_tokens(ratio, n),
             ckv_paged_freed_blocks(&pl, old_seq, new_seq));
    } else if (cmd == "attn_ws") {
      ckv_layout l = read_layout(in);
      int q_heads;
      in >> q_heads;
      size_t bytes = 0;
      const int st = ckv_decode_attn_workspace(&l, q_heads, &bytes);
      printf("attn_ws %d %zu\n", st, bytes);
    } else if (cmd == "compress_err") {         // argument errors of ckv_compress, found on the host before any launch
      ckv_layout l = read_layout(in), o = read_layout(in);
      ckv_params p = read_params(in);
      unsigned long long ws_bytes, k_addr;
      in >> ws_bytes >> k_addr;
      const int st = ckv_compress(reinterpret_cast<void*>(k_addr), fake, nullptr, &l, &p, reinterpret_cast<void*>(1ull << 40),
                                  reinterpret_cast<void*>(1ull << 41), reinterpret_cast<int32_t*>(1ull << 42), &o, nullptr,
                                  reinterpret_cast<void*>(1ull << 43), (size_t)ws_bytes, nullptr);
      printf("compress_err %d\n", st);
    } else if (cmd == "match_err") {
      ckv_layout l = read_layout(in);
      int chunk;
      in >> chunk;
      printf("match_err %d\n", ckv_match(nullptr, &l, chunk, reinterpret_cast<int32_t*>(fake), reinterpret_cast<float*>(fake), nullptr));
    } else {
      printf("unknown %s\n", cmd.c_str());
    }
  }
  printf("done %s | %s\n", ckv_version(), ckv_strerror(-4));
  return 0;
}
