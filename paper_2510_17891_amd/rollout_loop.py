"""Group rollout loop on top of the C boundary: G sampled outputs per prompt (Section 2.3), generated with
continuous batching inside a fixed KV pool.

This is the host step scheduler: it decides which groups are resident, which sequences are stepped, and when pages
go back to the pool.  Every arithmetic step (prefill, decode, sampling, log-probabilities) happens inside the
library; the loop only marshals ids and keeps views of the per-step output rows.

Scheduling never changes results: sequence (i, j) always has id i*G + j, its random stream is keyed by that id and
the token position, and the kernels are batch-invariant, so the tokens and log-probabilities are the same whatever
the pool size, admission order or batch composition.
"""
import torch

from .binding import RLError, RL_ERR_KV_FULL, _i32

KV_BLOCK = 16


def _pages(tokens):
    return (tokens + KV_BLOCK - 1) // KV_BLOCK


def group_page_need(prompt_len, new_tokens):
    """Pages a group holds at its largest: the prompt's full pages once, and per member the pages that its partial
    prompt page and its own tokens add.  The last sampled token is never fed back, so a member caches
    prompt_len + new - 1 tokens at most."""
    shared = prompt_len // KV_BLOCK
    return shared + sum(max(_pages(prompt_len + max(n, 1) - 1), _pages(prompt_len)) - shared for n in new_tokens)


def generate_groups(ro, prompts, group_size, max_new_tokens, temperature=1.0, seed=0, top_k=0, top_p=0.0,
                    eos_id=None, on_step=None):
    """Sample `group_size` outputs for every prompt.

    prompts         list of token-id lists
    max_new_tokens  int, or one int per sequence (len(prompts) * group_size, group-major): the length limit of
                    Appendix D, or pre-drawn lengths for synthetic workloads
    eos_id          stop a sequence after it samples this id (checked one call behind, from an asynchronous copy of the
                    sampled ids: nothing waits for the GPU inside the loop)
    on_step         optional callback(step_index, n_active) for progress reporting

    Returns (tokens, logprobs): per sequence a list of ids and a list of floats, group-major.
    Needs max_seqs >= len(prompts) * group_size; groups are admitted in order whenever the pool can hold them up
    to their length limit, so a decode step can never run out of pages; a group that cannot fit an empty pool
    raises RLError(RL_ERR_KV_FULL).
    """
    G = group_size
    n_seq = len(prompts) * G
    limits = [int(max_new_tokens)] * n_seq if isinstance(max_new_tokens, int) else [int(v) for v in max_new_tokens]
    assert len(limits) == n_seq and all(v >= 1 for v in limits)
    assert ro.cfg.max_seqs >= n_seq, "one sequence id per output is needed"
    max_rows = ro.cfg.max_rows
    assert G <= max_rows, "a group is prefilled in one call"
    dev = ro.device
    total_pages = ro.rl_kv_stats()[1]
    reserved = 0                       # pages promised to resident groups
    need = [group_page_need(len(p), limits[i * G:(i + 1) * G]) for i, p in enumerate(prompts)]
    next_group = 0
    members_left = {}                  # group -> sequences still running
    active = []                        # sequence ids in batch order
    dead = [0] * n_seq                 # decode step after which a sequence has reached its length limit
    next_dead = [1 << 62]              # the earliest of them among the active sequences
    calls = []                         # the decode calls of a step: (ids, ids as a C array); rebuilt when `active` changes
    rows_t, rows_lp, rows_ids = [], [], []   # per call: device outputs and the ids they belong to
    # End-token checks run one call behind: the tokens of a call are copied to pinned host memory without waiting, and
    # read when the next call has been enqueued.  A sequence that drew the end token therefore takes one step more than
    # it needs (inside its page reservation: it was below its limit); the surplus tokens are dropped at the end.
    pending = []                       # (ids, pinned host tokens, event)
    spare = []                         # pinned buffers and events to use again
    step = 0

    def admit():
        """Prefill waiting groups while the pool can hold them."""
        nonlocal next_group, reserved
        while next_group < len(prompts):
            g = next_group
            if need[g] > total_pages:
                raise RLError(RL_ERR_KV_FULL, f"group {g} needs {need[g]} pages, the pool has {total_pages}")
            if reserved + need[g] > total_pages:
                return
            ids = list(range(g * G, (g + 1) * G))
            tok, lp = ro.rl_prefill_groups(ids, G, [prompts[g]], temperature, seed, top_k=top_k, top_p=top_p)
            reserved += need[g]
            next_group += 1
            record(ids, tok, lp)
            members_left[g] = G
            active.extend(ids)
            calls.clear()
            for k in ids:                # the prefill gave token 1; decode step `step + n` gives token n + 1
                dead[k] = step + limits[k] - 1
            next_dead[0] = min(next_dead[0], min(dead[k] for k in ids))

    def record(ids, tok, lp):
        rows_t.append(tok)
        rows_lp.append(lp)
        rows_ids.append(ids)           # lists are never changed once they are in a call
        if eos_id is not None:
            buf, ev = spare.pop() if spare else (torch.empty(max_rows, dtype=torch.int32, pin_memory=True), torch.cuda.Event())
            buf[:len(ids)].copy_(tok, non_blocking=True)
            ev.record()
            pending.append((ids, buf, ev))

    def retire(finished):
        nonlocal reserved
        finished = [s for s in dict.fromkeys(finished) if s in running]
        if not finished:
            return
        ro.rl_free_seqs(finished)
        gone = set(finished)
        running.difference_update(gone)
        active[:] = [s for s in active if s not in gone]
        calls.clear()
        next_dead[0] = min((dead[s] for s in active), default=1 << 62)
        for s in finished:
            g = s // G
            members_left[g] -= 1
            if members_left[g] == 0:   # the reservation covers the group's shared pages until its last member leaves
                reserved -= need[g]
                del members_left[g]

    def at_limit(ids):
        if step < next_dead[0]:
            return []
        return [s for s in ids if step >= dead[s]]

    def drew_end_token(keep_last):
        """Sequences whose end token has arrived on the host; the newest `keep_last` copies stay in flight."""
        done = []
        while len(pending) > keep_last:
            ids, buf, ev = pending.pop(0)
            ev.synchronize()
            done += [s for s, t in zip(ids, buf[:len(ids)].tolist()) if t == eos_id]
            spare.append((buf, ev))
        return done

    running = set()
    while active or next_group < len(prompts):
        first = len(active)
        admit()
        running.update(active[first:])
        retire(at_limit(active[first:]))      # an output of one token ends with its prefill
        if not active:
            retire(drew_end_token(0))
            continue
        if not calls:
            for b0 in range(0, len(active), max_rows):
                ids = active[b0:b0 + max_rows]
                calls.append((ids, _i32(ids)))
        for ids, ids_c in calls:
            # in_tokens = None: the library feeds every sequence the token it returned for it last
            tok, lp = ro.rl_decode_step(ids_c, None, temperature, seed, top_k=top_k, top_p=top_p)
            record(ids, tok, lp)
        step += 1
        n_calls = len(calls)
        finished = at_limit(active)
        if eos_id is not None:
            finished += drew_end_token(n_calls)   # everything but the calls just enqueued
        retire(finished)
        if on_step is not None:
            on_step(step, len(active))

    torch.cuda.synchronize(dev)
    tokens = [[] for _ in range(n_seq)]
    logprobs = [[] for _ in range(n_seq)]
    all_t = torch.cat(rows_t).cpu().tolist() if rows_t else []
    all_lp = torch.cat(rows_lp).cpu().tolist() if rows_lp else []
    k = 0
    for ids in rows_ids:
        for s in ids:
            if len(tokens[s]) < limits[s] and not (eos_id is not None and tokens[s] and tokens[s][-1] == eos_id):
                tokens[s].append(all_t[k])
                logprobs[s].append(all_lp[k])
            k += 1
    return tokens, logprobs
