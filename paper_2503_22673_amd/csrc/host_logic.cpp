// Host-only half of the C interface: configuration checks, the packing plan and the segment-table check.
// No GPU call and no HIP header in this file, so that it can also be built with a host compiler and its
// sanitizers (tests/test_host_sanitizer.py does that and drives it with valid and invalid inputs).
#include "host_logic.h"
#include <stdarg.h>
#include <stdio.h>
#include <algorithm>

static int host_fail(std::string* err, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap; va_start(ap, fmt); vsnprintf(buf, sizeof buf, fmt, ap); va_end(ap);
  if (err) *err = buf;
  return code;
}


int check_config(const as_model_config* c, std::string* err) {
  if (c->struct_size != sizeof(as_model_config)) return host_fail(err, AS_ERR_CONFIG, "struct_size %u != %zu", c->struct_size, sizeof(as_model_config));
  if (c->n_layers < 1 || c->d_model < 1 || c->ffn < 1 || c->vocab < 2) return host_fail(err, AS_ERR_CONFIG, "non-positive model size");
  if (c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads) return host_fail(err, AS_ERR_CONFIG, "n_q_heads must be a positive multiple of n_kv_heads");
  if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128) return host_fail(err, AS_ERR_CONFIG, "head_dim must be 32, 64 or 128");
  if (c->mode != AS_FP32 && c->mode != AS_BF16) return host_fail(err, AS_ERR_CONFIG, "mode");
  if (c->train_mode != AS_LORA && c->train_mode != AS_FULL) return host_fail(err, AS_ERR_CONFIG, "train_mode");
  if (!(c->rms_eps > 0.f) || !(c->rope_base > 1.f)) return host_fail(err, AS_ERR_CONFIG, "rms_eps / rope_base");
  const bool moe = c->n_experts != 0 || c->top_k != 0;
  if (moe) {
    if (c->n_experts < 8 || c->n_experts > 64 || c->n_experts % 8) return host_fail(err, AS_ERR_CONFIG, "n_experts must be a multiple of 8 in [8, 64]");
    if (c->top_k != 2) return host_fail(err, AS_ERR_CONFIG, "top_k must be 2");
    if (c->train_mode != AS_LORA) return host_fail(err, AS_ERR_CONFIG, "mixture-of-experts models are trained with adapters only");
    if (c->lora_targets & 0x70u) return host_fail(err, AS_ERR_CONFIG, "adapters on expert projections are not supported");
  }
  if (c->train_mode == AS_LORA) {
    if (c->lora_rank < 1 || c->lora_rank > 256) return host_fail(err, AS_ERR_CONFIG, "lora_rank must be in [1, 256]");
    if (!(c->lora_targets & 0xff)) return host_fail(err, AS_ERR_CONFIG, "LoRA mode needs at least one target");
    if (c->lora_targets & ~0xffu) return host_fail(err, AS_ERR_CONFIG, "unknown adapter target");
    if (!moe && (c->lora_targets & 0x80u)) return host_fail(err, AS_ERR_CONFIG, "router adapters need a mixture-of-experts model");
  } else if (c->lora_rank != 0 || c->lora_targets != 0) {
    return host_fail(err, AS_ERR_CONFIG, "full fine-tuning takes no adapters");
  }
  if (c->recompute < 0 || c->recompute > 2) return host_fail(err, AS_ERR_CONFIG, "recompute must be 0, 1 or 2");
  if (c->weight_format != AS_W_DENSE && c->weight_format != AS_W_NF4) return host_fail(err, AS_ERR_CONFIG, "weight_format");
  if (c->weight_format == AS_W_NF4) {
    if (c->train_mode != AS_LORA || moe) return host_fail(err, AS_ERR_CONFIG, "NF4 weights are a frozen dense base: LoRA mode, no experts");
    if (c->d_model % 64 || c->ffn % 64 || (c->n_q_heads * c->head_dim) % 64 || (c->n_kv_heads * c->head_dim) % 64)
      return host_fail(err, AS_ERR_CONFIG, "NF4 weights need widths that are multiples of the 64-element block");
  }
  return AS_OK;
}


// Host half of packing: validation, next-fit row assignment, piece list and
// segment table.  Touches no GPU state, so it can be tested without one.
int pack_plan(int vocab, const int32_t* turn_tokens, const int32_t* turn_offsets,
              const uint8_t* turn_roles, const int32_t* traj_offsets, int32_t n_traj,
                     int32_t T, int32_t max_rows, int32_t truncate, int32_t policy, std::vector<Piece>& pieces,
                     std::vector<int32_t>& cu, std::vector<uint8_t>& skip, int32_t* n_rows, int32_t* n_consumed,
                     int32_t* traj_row, std::string* err) {
  if (T <= 0 || max_rows < 0 || n_traj < 0) return host_fail(err, AS_ERR_SHAPE, "as_pack: row_len must be positive, counts non-negative");
  if (policy != AS_PACK_NEXT_FIT && policy != AS_PACK_BEST_FIT_DECREASING) return host_fail(err, AS_ERR_SHAPE, "as_pack: unknown policy %d", policy);
  if ((int64_t)T * max_rows > INT32_MAX) return host_fail(err, AS_ERR_SHAPE, "as_pack: max_rows*row_len exceeds int32");
  if (traj_offsets[0] != 0 || turn_offsets[0] != 0) return host_fail(err, AS_ERR_SHAPE, "as_pack: offsets must start at 0");
  // both offset tables are checked in full before any token is read: the last turn offset is the
  // length of turn_tokens, and no earlier offset may point past it
  for (int32_t i = 0; i < n_traj; i++)
    if (traj_offsets[i + 1] < traj_offsets[i]) return host_fail(err, AS_ERR_SHAPE, "as_pack: traj_offsets must not decrease (trajectory %d)", i);
  for (int32_t t = 0, nt = traj_offsets[n_traj]; t < nt; t++)
    if (turn_offsets[t + 1] < turn_offsets[t]) return host_fail(err, AS_ERR_SHAPE, "as_pack: turn_offsets must not decrease (turn %d)", t);
  pieces.clear(); cu.clear(); cu.push_back(0); skip.clear();
  // roles and token ids of trajectory i, and its length cut to a row
  auto measure = [&](int32_t i, int32_t* len) -> int {
    int64_t L = 0;
    for (int32_t t = traj_offsets[i]; t < traj_offsets[i + 1]; t++) {
      if (turn_roles[t] > AS_ROLE_TOOL) return host_fail(err, AS_ERR_ROLE, "as_pack: role code %d of turn %d is outside 0..3", (int)turn_roles[t], t);
      for (int32_t k = turn_offsets[t]; k < turn_offsets[t + 1]; k++)
        if (turn_tokens[k] < 0 || turn_tokens[k] >= vocab)
          return host_fail(err, AS_ERR_TOKEN_RANGE, "as_pack: token %d at offset %d is outside [0, %d)", turn_tokens[k], k, vocab);
      L += turn_offsets[t + 1] - turn_offsets[t];
    }
    if (L > T) {
      if (!truncate) return host_fail(err, AS_ERR_TOO_LONG, "as_pack: trajectory %d has %lld tokens, row_len is %d", i, (long long)L, T);
      L = T;
    }
    *len = (int32_t)L;
    return AS_OK;
  };
  // the first L tokens of trajectory i as one segment at `fill` of row `row`
  auto emit = [&](int32_t i, int32_t L, int32_t row, int32_t fill) {
    int32_t left = L; bool any_loss = false;
    for (int32_t t = traj_offsets[i]; t < traj_offsets[i + 1] && left > 0; t++) {
      int32_t len = std::min(turn_offsets[t + 1] - turn_offsets[t], left);
      if (len <= 0) continue;
      pieces.push_back({row * T + fill, turn_offsets[t], (uint8_t)(turn_roles[t] == AS_ROLE_ASSISTANT)});
      any_loss = any_loss || turn_roles[t] == AS_ROLE_ASSISTANT;
      fill += len; left -= len;
    }
    cu.push_back(row * T + fill); skip.push_back(any_loss ? 0 : 1);
  };
  auto pad_tail = [&](int32_t row, int32_t fill) {
    if (fill < T) { pieces.push_back({row * T + fill, -1, 0}); cu.push_back((row + 1) * T); skip.push_back(1); }
  };
  int rc;
  if (policy == AS_PACK_NEXT_FIT) {
    int32_t fill = 0, rows = 0, consumed = 0; bool open = false;
    for (int32_t i = 0; i < n_traj && rows < max_rows; i++) {
      int32_t L;
      if ((rc = measure(i, &L))) return rc;
      if (L == 0) { consumed++; if (traj_row) traj_row[i] = -2; continue; }
      if (open && fill + L > T) { pad_tail(rows, fill); rows++; fill = 0; open = false; if (rows >= max_rows) break; }
      open = true;
      emit(i, L, rows, fill);
      if (traj_row) traj_row[i] = rows;
      fill += L; consumed++;
      if (fill == T) { rows++; fill = 0; open = false; }
    }
    if (open) { pad_tail(rows, fill); rows++; }
    if (traj_row) for (int32_t i = consumed; i < n_traj; i++) traj_row[i] = -1;
    *n_rows = rows; *n_consumed = consumed;
    return AS_OK;
  }
  // Best fit decreasing: by non-increasing length (ties in input order), each trajectory into the open row
  // it fills best (least free space left, ties to the lowest row); a new row only when none has room; with
  // max_rows rows open and no room the trajectory is left out.
  std::vector<int32_t> len(n_traj), order, place(n_traj, -1);
  for (int32_t i = 0; i < n_traj; i++) {
    if ((rc = measure(i, &len[i]))) return rc;
    if (len[i] > 0) order.push_back(i); else place[i] = -2;
  }
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return len[a] > len[b]; });
  std::vector<std::vector<int32_t>> members;
  std::vector<int32_t> free_;
  for (int32_t i : order) {
    int best = -1;
    for (int r = 0; r < (int)members.size(); r++)
      if (free_[r] >= len[i] && (best < 0 || free_[r] < free_[best])) best = r;
    if (best < 0) {
      if ((int32_t)members.size() >= max_rows) continue;
      members.emplace_back(); free_.push_back(T);
      best = (int)members.size() - 1;
    }
    members[best].push_back(i); free_[best] -= len[i]; place[i] = best;
  }
  int32_t consumed = 0;
  for (int32_t i = 0; i < n_traj; i++) { consumed += place[i] != -1; if (traj_row) traj_row[i] = place[i]; }
  for (int32_t r = 0; r < (int32_t)members.size(); r++) {
    int32_t fill = 0;
    for (int32_t i : members[r]) { emit(i, len[i], r, fill); fill += len[i]; }
    pad_tail(r, fill);
  }
  *n_rows = (int32_t)members.size(); *n_consumed = consumed;
  return AS_OK;
}


int check_cu(const int32_t* cu, int32_t S, int64_t N, int32_t T, int* max_seg, std::string* err) {
  if (S < 1) return host_fail(err, AS_ERR_CU_SEQLENS, "cu_seqlens: at least one segment is needed");
  if (cu[0] != 0) return host_fail(err, AS_ERR_CU_SEQLENS, "cu_seqlens[0] = %d, must be 0", cu[0]);
  if (cu[S] != N) return host_fail(err, AS_ERR_CU_SEQLENS, "cu_seqlens[%d] = %d, must be n_rows*row_len = %lld", S, cu[S], (long long)N);
  int mx = 0;
  for (int s = 0; s < S; s++) {
    if (cu[s + 1] <= cu[s]) return host_fail(err, AS_ERR_CU_SEQLENS, "cu_seqlens not strictly increasing at %d", s);
    if (cu[s] / T != (cu[s + 1] - 1) / T) return host_fail(err, AS_ERR_CU_SEQLENS, "segment %d crosses a row end", s);
    mx = std::max(mx, cu[s + 1] - cu[s]);
  }
  *max_seg = mx;
  return AS_OK;
}

