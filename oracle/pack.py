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

A second policy, ``best_fit_decreasing`` (the classical bin-packing heuristic of that name), cuts the
pad share when a pool of trajectories larger than one batch is on offer: the non-empty trajectories
(over-long ones cut to ``row_len`` first) are taken by non-increasing length, ties in input order; each
goes to the open row whose free space after placing it is smallest (ties: the lowest row), a new row is
opened only when no open row has room, and when ``max_rows`` rows are open and none has room the
trajectory is left out (``traj_row`` -1: offer it again with the next batch).  Rows are written in row
order, the trajectories of a row in the order they were placed; masks, tails and ``cu_seqlens`` as above.
All trajectories are validated, placed or not.

Everything is done one token at a time on purpose.
"""
import numpy as np

ROLE_SYSTEM, ROLE_USER, ROLE_ASSISTANT, ROLE_TOOL = 0, 1, 2, 3


class PackError(ValueError):
    pass


def _flatten(traj, vocab):
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
    return flat_tok, flat_msk


def _pack_best_fit_decreasing(trajectories, T, max_rows, pad_id, truncate, vocab):
    flat = []
    for traj in trajectories:
        tok, msk = _flatten(traj, vocab)
        if len(tok) > T:
            if not truncate:
                raise PackError("too long")
            tok, msk = tok[:T], msk[:T]
        flat.append((tok, msk))
    traj_row = [-2 if len(tok) == 0 else -1 for tok, _ in flat]      # -2: empty, consumed without trace
    order = sorted([i for i in range(len(flat)) if len(flat[i][0]) > 0], key=lambda i: (-len(flat[i][0]), i))
    rows, free = [], []                                              # members of each open row, its free space
    for i in order:
        L = len(flat[i][0])
        best = -1
        for r in range(len(rows)):
            if free[r] >= L and (best < 0 or free[r] < free[best]):
                best = r
        if best < 0:
            if len(rows) >= max_rows:
                continue
            rows.append([]); free.append(T)
            best = len(rows) - 1
        rows[best].append(i); free[best] -= L; traj_row[i] = best
    tokens, mask, cu = [], [], [0]
    for members in rows:
        for i in members:
            tokens.extend(flat[i][0]); mask.extend(flat[i][1]); cu.append(len(tokens))
        if len(tokens) % T:
            for _ in range(T - len(tokens) % T):
                tokens.append(pad_id); mask.append(0)
            cu.append(len(tokens))
    return dict(tokens=np.asarray(tokens, dtype=np.int32).reshape(-1),
                cu_seqlens=np.asarray(cu, dtype=np.int32),
                loss_mask=np.asarray(mask, dtype=np.uint8).reshape(-1),
                n_rows=len(rows), n_segments=len(cu) - 1,
                n_traj_consumed=sum(1 for r in traj_row if r != -1),
                traj_row=np.asarray(traj_row, dtype=np.int32))


def pack(trajectories, row_len, max_rows, pad_id=0, truncate=True, vocab=None, policy="next_fit"):
    """trajectories: list of trajectories; a trajectory is a list of turns;
    a turn is (role, sequence of token ids).

    Returns dict(tokens int32[R*T], cu_seqlens int32[S+1], loss_mask
    uint8[R*T], n_rows, n_segments, n_traj_consumed); with policy
    "best_fit_decreasing" also traj_row int32[n_traj] (row of each trajectory,
    -1 = left out, -2 = empty) and n_traj_consumed counts placed + empty.
    """
    T = int(row_len)
    if T <= 0 or max_rows < 0:
        raise PackError("shape")
    if policy == "best_fit_decreasing":
        return _pack_best_fit_decreasing(trajectories, T, max_rows, pad_id, truncate, vocab)
    if policy != "next_fit":
        raise PackError("policy")
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
