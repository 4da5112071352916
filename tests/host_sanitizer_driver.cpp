// Driver for the host-only logic of the C interface (csrc/host_logic.cpp) under AddressSanitizer and
// UndefinedBehaviorSanitizer.  Reads cases from stdin, one per block, and prints what the functions return;
// tests/test_host_sanitizer.py writes the cases (valid ones from the float64 reference's packer, invalid ones by
// hand) and checks the answers.  Every input array is a heap block of exactly its stated length, so that a read
// past an offset table or a token array is reported.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <memory>
#include "host_logic.h"

template <typename T> static std::unique_ptr<T[]> read_array(int n) {
  std::unique_ptr<T[]> a(new T[n > 0 ? n : 0]);          // n == 0: a zero-length block, any read is out of bounds
  for (int i = 0; i < n; i++) { long long v; if (scanf("%lld", &v) != 1) exit(3); a[i] = (T)v; }
  return a;
}

int main() {
  char kind[32];
  while (scanf("%31s", kind) == 1) {
    std::string err;
    if (!strcmp(kind, "pack")) {
      int vocab, T, max_rows, truncate, policy, n_traj, n_turns, n_tok;
      if (scanf("%d %d %d %d %d %d %d %d", &vocab, &T, &max_rows, &truncate, &policy, &n_traj, &n_turns, &n_tok) != 8) return 3;
      auto traj_offsets = read_array<int32_t>(n_traj + 1);
      auto turn_offsets = read_array<int32_t>(n_turns + 1);
      auto turn_roles = read_array<uint8_t>(n_turns);
      auto turn_tokens = read_array<int32_t>(n_tok);
      std::vector<Piece> pieces; std::vector<int32_t> cu; std::vector<uint8_t> skip;
      std::unique_ptr<int32_t[]> traj_row(new int32_t[n_traj > 0 ? n_traj : 0]);
      int32_t rows = 0, consumed = 0;
      const int rc = pack_plan(vocab, turn_tokens.get(), turn_offsets.get(), turn_roles.get(), traj_offsets.get(), n_traj, T, max_rows,
                               truncate, policy, pieces, cu, skip, &rows, &consumed, traj_row.get(), &err);
      printf("rc %d\n", rc);
      if (rc) { printf("err %s\n", err.c_str()); continue; }
      printf("rows %d consumed %d\n", rows, consumed);
      printf("cu"); for (int32_t v : cu) printf(" %d", v); printf("\n");
      printf("skip"); for (uint8_t v : skip) printf(" %d", (int)v); printf("\n");
      printf("traj_row"); for (int i = 0; i < n_traj; i++) printf(" %d", traj_row[i]); printf("\n");
      // the packed stream the pieces describe (what the device kernel writes): token, or -1 for pad; mask bit
      const int64_t n_out = (int64_t)rows * T;
      std::vector<int32_t> tok(n_out, -1); std::vector<int> msk(n_out, 0);
      for (size_t i = 0; i < pieces.size(); i++) {
        const int64_t end = i + 1 < pieces.size() ? pieces[i + 1].dst : n_out;
        for (int64_t d = pieces[i].dst; d < end; d++) {
          if (d < 0 || d >= n_out) { printf("piece out of range\n"); return 4; }
          if (pieces[i].src >= 0) {
            const int64_t sidx = pieces[i].src + (d - pieces[i].dst);
            if (sidx < 0 || sidx >= n_tok) { printf("source out of range\n"); return 4; }
            tok[d] = turn_tokens[sidx]; msk[d] = pieces[i].mask;
          }
        }
      }
      printf("tokens"); for (int32_t v : tok) printf(" %d", v); printf("\n");
      printf("mask"); for (int v : msk) printf(" %d", v); printf("\n");
    } else if (!strcmp(kind, "cu")) {
      int S; long long N; int T;
      if (scanf("%d %lld %d", &S, &N, &T) != 3) return 3;
      auto cu = read_array<int32_t>(S + 1 > 0 ? S + 1 : 0);
      int max_seg = -1;
      const int rc = check_cu(cu.get(), S, N, T, &max_seg, &err);
      printf("rc %d max_seg %d\n", rc, rc ? -1 : max_seg);
    } else if (!strcmp(kind, "cfg")) {
      as_model_config c; memset(&c, 0, sizeof c);
      int v[16]; float f[3];
      if (scanf("%d %d %d %d %d %d %d %d %d %d %f %f %d %f %d %d %d %d %d", &v[0], &v[1], &v[2], &v[3], &v[4], &v[5], &v[6], &v[7], &v[8], &v[9],
                &f[0], &f[1], &v[10], &f[2], &v[11], &v[12], &v[13], &v[14], &v[15]) != 19) return 3;
      c.struct_size = (uint32_t)v[0]; c.n_layers = v[1]; c.d_model = v[2]; c.n_q_heads = v[3]; c.n_kv_heads = v[4]; c.head_dim = v[5];
      c.ffn = v[6]; c.vocab = v[7]; c.n_experts = v[8]; c.top_k = v[9]; c.rms_eps = f[0]; c.rope_base = f[1]; c.lora_rank = v[10];
      c.lora_alpha = f[2]; c.lora_targets = (uint32_t)v[11]; c.mode = v[12]; c.train_mode = v[13]; c.recompute = v[14]; c.weight_format = v[15];
      if (c.struct_size == 0) c.struct_size = sizeof(as_model_config);
      printf("rc %d\n", check_config(&c, &err));
    } else {
      return 3;
    }
  }
  return 0;
}
