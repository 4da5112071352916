// Host-only logic of the C interface (see host_logic.cpp): no HIP types here.
#pragma once
#include <stdint.h>
#include <string>
#include <vector>
#include "actionstudio.h"

// one run of tokens of the packed stream: destination offset, source offset in turn_tokens (-1: pad), mask bit
struct Piece { int32_t dst, src; uint8_t mask; };

// Every function returns AS_OK or a negative as_status and, on failure, a message in *err.
int check_config(const as_model_config* c, std::string* err);
// Validation, row assignment (policy), piece list, segment table and loss-free-segment flags of as_pack / as_pack_policy.
int pack_plan(int vocab, const int32_t* turn_tokens, const int32_t* turn_offsets,
              const uint8_t* turn_roles, const int32_t* traj_offsets, int32_t n_traj,
              int32_t T, int32_t max_rows, int32_t truncate, int32_t policy, std::vector<Piece>& pieces,
              std::vector<int32_t>& cu, std::vector<uint8_t>& skip, int32_t* n_rows, int32_t* n_consumed,
              int32_t* traj_row, std::string* err);
// cu[0..S] is a partition of [0, N) into segments none of which crosses a multiple of T; *max_seg = longest segment
int check_cu(const int32_t* cu, int32_t S, int64_t N, int32_t T, int* max_seg, std::string* err);
