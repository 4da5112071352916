"""Reference packer: trajectories -> (tokens, cu_seqlens, loss_mask).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this
module; only the tests, the smoke check and the CPU-baseline leg of the
benchmark do.

What is computed follows the paper's Section 3.2.1 (Universal Data Parser:
every element of a conversation is encoded on its own so that a loss mask
can be attached per element) and the role vocabulary of Unified Format 2.0
(Appendix, "Unified Format 2.0": system, user, assistant, tool).  The
packing policy itself is not in the paper; the policy coded here is the
definition both sides are held to:

* trajectories are taken in input order; a trajectory's length is the sum
  of its turn lengths; zero-length trajectories are consumed and leave no
  trace;
* next-fit: a trajectory that does not fit behind the current fill of the
  open row closes that row (its tail is filled with ``pad_id``) and opens
  the next one;
* a trajectory longer than a row keeps its first ``row_len`` tokens when
  ``truncate`` is set and is an error otherwise;
* packing stops when ``max_rows`` rows are closed or the input is used up;
* ``loss_mask[t] = 1`` exactly for tokens that came from an assistant turn;
* ``cu_seqlens`` partitions the flat stream [0, n_rows*row_len): one entry
  per trajectory end, and every non-empty pad tail is a segment of its own.

Everything is done one token at a time on purpose.
"""
import numpy as np

ROLE_SYSTEM, ROLE_USER, ROLE_ASSISTANT, ROLE_TOOL = 0, 1, 2, 3


class PackError(ValueError):
    pass


def pack(trajectories, row_len, max_rows, pad_id=0, truncate=True, vocab=None):
    """trajectories: list of trajectories; a trajectory is a list of turns;
    a turn is (role, sequence of token ids).

    Returns dict(tokens int32[R*T], cu_seqlens int32[S+1], loss_mask
    uint8[R*T], n_rows, n_segments, n_traj_consumed).
    """
    T = int(row_len)
    if T <= 0 or max_rows < 0:
        raise PackError("shape")
    tokens, mask, cu = [], [], [0]
    fill = 0            # tokens already placed in the open row
    rows_closed = 0
    row_open = False
    consumed = 0

    def close_row():
        nonlocal fill, rows_closed, row_open
        if fill < T:
            for _ in range(T - fill):
                tokens.append(pad_id)
                mask.append(0)
            cu.append(len(tokens))
        rows_closed += 1
        fill = 0
        row_open = False

    for traj in trajectories:
        if rows_closed >= max_rows:
            break
        flat_tok, flat_msk = [], []
        for role, toks in traj:
            if role not in (ROLE_SYSTEM, ROLE_USER, ROLE_ASSISTANT, ROLE_TOOL):
                raise PackError("role")
            for tk in toks:
                tk = int(tk)
                if tk < 0 or (vocab is not None and tk >= vocab):
                    raise PackError("token range")
                flat_tok.append(tk)
                flat_msk.append(1 if role == ROLE_ASSISTANT else 0)
        L = len(flat_tok)
        if L == 0:
            consumed += 1
            continue
        if L > T:
            if not truncate:
                raise PackError("too long")
            flat_tok, flat_msk, L = flat_tok[:T], flat_msk[:T], T
        if row_open and fill + L > T:
            close_row()
            if rows_closed >= max_rows:
                break
        row_open = True
        tokens.extend(flat_tok)
        mask.extend(flat_msk)
        fill += L
        cu.append(len(tokens))
        consumed += 1
        if fill == T:
            # the row is exactly full: it closes without a pad segment
            rows_closed += 1
            fill = 0
            row_open = False
    if row_open:
        close_row()
    n_rows = rows_closed
    assert len(tokens) == n_rows * T
    return dict(tokens=np.asarray(tokens, dtype=np.int32).reshape(-1),
                cu_seqlens=np.asarray(cu, dtype=np.int32),
                loss_mask=np.asarray(mask, dtype=np.uint8).reshape(-1),
                n_rows=n_rows, n_segments=len(cu) - 1,
                n_traj_consumed=consumed)
