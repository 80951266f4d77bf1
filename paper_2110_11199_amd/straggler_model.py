"""Wall-clock model of the paper's slow-learner experiment (Section IV-D, the straggler table) on one GPU.

In the paper one of 16 learners is put to sleep so that a minibatch takes it 5, 10 or 100 times as long as the
others; the ring variants (fixed and random mixing) go on without it, delay-by-one and synchronous SGD wait
for it.  Here the learners are replicas on one GPU, so "a learner's gradient computation on its own device" is
stood in for by an idle kernel of a set duration (`adpsgd_delay`): one per iteration for the L-1 ordinary
learners together (they run side by side in the paper), a longer one for the slow learner, on streams of their
own.  Per iteration the host
  * starts the idle kernels of the learners that are not still busy,
  * waits for the ordinary learners; in the ring variants it then only LOOKS whether the slow learner has
    finished (an event query) and, if not, runs the iteration without it (`adpsgd_step_masked`: the learner is
    the iteration's straggler, its model stays as it is, its ring partner mixes with nobody); in the
    synchronous variants (delay-by-one, synchronous SGD) it waits for the slow learner too,
  * runs mixing and update.
What comes out: wall-clock per iteration and per "epoch" (a fixed number of learner minibatches, the paper's
measure), the masks that were realised (any of them is a valid run of the method: the test replays them through
the oracle), all on the model-free workload (flat parameter vectors, a fixed gradient per learner).

No method arithmetic here: schedule, mixing and update run in the library.
"""
import time


_STREAMS = None


def _concurrent_streams():
    """Two streams whose kernels run side by side, and beside the current stream.  HIP multiplexes its streams
    over a few hardware queues and two streams that share a queue run their kernels one after the other, which
    would make everybody wait for the slow learner whatever the method does: candidates are therefore tried
    (a long idle kernel on one, a short one on the other, timed) until a pair overlaps."""
    global _STREAMS
    if _STREAMS is not None:
        return _STREAMS
    import torch
    from . import binding as Bd
    main = torch.cuda.current_stream()

    def blocked_by(long_stream, short_stream):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        Bd.adpsgd_delay(6000, long_stream.cuda_stream)
        Bd.adpsgd_delay(200, short_stream.cuda_stream)
        short_stream.synchronize()
        dt = time.perf_counter() - t0
        torch.cuda.synchronize()
        return dt > 3e-3
    cand = [torch.cuda.Stream() for _ in range(8)]
    for i, s_slow in enumerate(cand):
        if blocked_by(s_slow, main):
            continue
        for s_fast in cand[i + 1:]:
            if not blocked_by(s_slow, s_fast) and not blocked_by(s_fast, main):
                _STREAMS = (s_fast, s_slow)
                return _STREAMS
    raise RuntimeError("no two streams of this process run their kernels concurrently")


def run(pattern, L, P, factor, iterations, grad_us, seed=0, lr=0.1, slow=0, device="cuda:0", x0=None, grads=None):
    """One run.  pattern: binding.FIXED_RING / RANDOM_RING (asynchronous) or D1D / SDPSGD (wait for everybody).
    factor: how many times longer the slow learner's minibatch takes (1 = no straggler).
    Returns a dict: seconds, iterations, masks (list of L flags per iteration), learner_batches, engine."""
    import torch
    from . import binding as Bd
    torch.cuda.set_device(device)
    eng = Bd.Adpsgd(Bd.make_config(L, pattern, seed=seed, flat_params=P), device)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    if grads is None:
        grads = [torch.empty(P, device=device).normal_(0.0, 1e-3, generator=gen) for _ in range(L)]
    for i in range(L):
        eng.set_params(i, x0[i] if x0 is not None else torch.empty(P, device=device).uniform_(-0.05, 0.05, generator=gen))
    waits_for_all = pattern in (Bd.D1D, Bd.SDPSGD)
    main = torch.cuda.current_stream()
    s_fast, s_slow = _concurrent_streams()
    ev_fast, ev_slow, ev_upd = torch.cuda.Event(), torch.cuda.Event(), torch.cuda.Event()
    ev_upd.record(main)
    slow_busy = False
    masks, batches = [], 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(iterations):
        if not slow_busy:                     # the slow learner starts its next minibatch from the model it has now
            s_slow.wait_event(ev_upd)
            Bd.adpsgd_delay(int(grad_us * factor), s_slow.cuda_stream)
            ev_slow.record(s_slow)
            slow_busy = True
        s_fast.wait_event(ev_upd)
        Bd.adpsgd_delay(int(grad_us), s_fast.cuda_stream)
        ev_fast.record(s_fast)
        ev_fast.synchronize()                 # the ordinary learners have their gradients
        if waits_for_all or factor <= 1:      # no straggler: the "slow" learner is one of the ordinary ones
            ev_slow.synchronize()
            ready = True
        else:
            ready = ev_slow.query()           # a look, not a wait
        active = [1] * L
        if not ready:
            active[slow] = 0
        else:
            slow_busy = False
        eng.step(grads, lr, active=None if waits_for_all else active)
        ev_upd.record(main)
        masks.append(active)
        batches += sum(active)
    main.synchronize()                        # the last update is done (a slow learner may still be busy: nobody waits for it)
    seconds = time.perf_counter() - t0
    torch.cuda.synchronize()
    return {"seconds": seconds, "iterations": iterations, "masks": masks, "learner_batches": batches, "engine": eng,
            "grads": grads}


def slowdown_table(L=16, P=1 << 22, iterations=40, grad_us=2000, factors=(1, 5, 10, 100)):
    """Per pattern and delay factor: seconds per iteration and per L learner minibatches ("epoch" measure),
    both relative to the run without a straggler."""
    from . import binding as Bd
    out = {}
    for name, pattern in (("fixed_ring", Bd.FIXED_RING), ("random_ring", Bd.RANDOM_RING), ("delay_by_one", Bd.D1D)):
        rows = {}
        base_iter = base_epoch = None
        for f in factors:
            its = iterations if f < 100 or pattern != Bd.D1D else max(4, iterations // 10)      # 100x on a waiting variant is slow
            r = run(pattern, L, P, f, its, grad_us)
            r["engine"].close()
            per_iter = r["seconds"] / r["iterations"]
            per_epoch = r["seconds"] / r["learner_batches"] * L       # time per L learner minibatches
            if f == 1:
                base_iter, base_epoch = per_iter, per_epoch
            rows["%dx" % f] = {"ms_per_iteration": per_iter * 1e3, "slowdown_per_iteration": per_iter / base_iter,
                               "slowdown_per_epoch": per_epoch / base_epoch,
                               "straggler_took_part_in": sum(m[0] for m in r["masks"]), "iterations": r["iterations"]}
        out[name] = rows
    return out
