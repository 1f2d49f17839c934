"""GPU parity over the FULL lengths of the three long workloads (section 4.3: the memory and the cost of
a step stay constant once the stream is longer than the capacity M, and the section 3.4 sum keeps
growing without decay in bf16 storage):

    cfg3  one layer of the Llama-shaped stack: 2 x 512 prompt tokens through bct_prefill, then 8192 decode steps
    cfg4  GQA (32 query / 8 KV heads), M = 8192: 16384 decode steps
    cfg5  M = 16384: 4 x 512 prompt tokens through bct_prefill, then 65536 decode steps

The GPU runs the whole trajectory at the full shape, in the launch configuration bench.py times.  The
oracle cannot (10^14 to 10^15 element updates), so it watches in three ways, each on a sample of the
(batch element, KV head) memories, which are independent of one another (pinned on the oracle):

  lock-step   the first 64 decode steps: the oracle steps freely beside the GPU from a common state,
              every output compared;
  resync      at steps M-1, M, M+1, 2M, eight seeded random steps and the last one: the GPU's state
              is loaded into the oracle, both take that one step on the same inputs, the output and
              the new state are compared (per-step parity at any depth); every prompt chunk is checked
              the same way;
  replica     a free-running oracle that never sees the GPU's state follows a few memories from the
              first token for as many steps as the oracle's speed allows (all 8192 of cfg3; the first
              1024 of cfg4 and cfg5, where an oracle step of 8 memories takes 27-36 ms): its outputs
              are compared at every step and the drift of the stored state is printed at intervals.

Inputs: the prompt, the lock-step and resync steps and every input of the replica's memories come from
bct_synth; the other inputs of the other steps, which no oracle ever reads, are N(0,1) drawn on the
device by torch's seeded generator (generating 65536 full steps on the host would take ten minutes).
"""
import concurrent.futures
import os

import numpy as np
import pytest

import bct_synth as syn
from _util import bf16_ulp, f64, to_dev, to_np, torch_dtype
from test_gpu_parity import check_out, check_state_one_step
from test_gpu_prefill import check_prefill_out, check_prefill_state, prefill_mass

pytestmark = pytest.mark.gpu

BLOCK = 256      # decode steps whose inputs are drawn on the device at once


@pytest.fixture(scope="module")
def P():
    import torch
    assert torch.cuda.is_available()
    import paper_2411_15785_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def R():
    from oracle import bct_ref
    return bct_ref


def _progress(line):
    print(line, flush=True)
    path = os.environ.get("BCT_TEST_PROGRESS_LOG")     # a file to append to, for runs whose stdout is captured
    if path:
        with open(path, "a") as f:
            f.write(line + "\n")


def unit_inputs(w, step, b, h0, nh, T=0):
    """(q, wq, wv) of the memories (b, h0 .. h0+nh-1) at global step `step`, drawn exactly as
    bct_synth.make_step draws them inside the full tensors (the generator is counter-based).
    T > 0: a chunk, [1][T][heads][d]; else [1][heads][d]."""
    s, G, d = syn.layer_seed(0), w.G, w.d

    def one(t):
        q = syn.normal(s, syn.TID_Q, t, (nh * G, d), start=(b * w.Hq + h0 * G) * d)
        wq = syn.normal(s, syn.TID_WQ, t, (nh, d), start=(b * w.Hkv + h0) * d)
        wv = syn.normal(s, syn.TID_WV, t, (nh, d), start=(b * w.Hkv + h0) * d)
        return [syn.pack(a, w.dtype) for a in (q, wq, wv)]

    if T == 0:
        return tuple(a[None] for a in one(step))
    toks = [one(step + t) for t in range(T)]
    return tuple(np.ascontiguousarray(np.stack([tk[i] for tk in toks], axis=0)[None]) for i in range(3))


def chunk_inputs(w, step, T):
    """bct_synth.make_step for a chunk, its T independent tokens drawn by a few threads."""
    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as ex:
        toks = list(ex.map(lambda t: syn.make_step(w, step + t), range(T)))
    return tuple(np.ascontiguousarray(np.stack([tk[i] for tk in toks], axis=1)) for i in range(3))


class Units:
    """A sample of memories: batch element b, KV heads h0 .. h0+NH-1, as a small oracle cache."""

    def __init__(self, R, w, mk, b, h0, nh):
        self.w, self.b, self.h0, self.nh = w, b, h0, nh
        self.ref = R.RefCache(w.M, 1, nh * w.G, nh, w.d, w.dtype, w.scale, w.scale)
        self.mk = np.ascontiguousarray(mk[h0:h0 + nh])
        self.ref.set_keys(self.mk)

    def cut(self, q, wq, wv):
        """The sample's rows of full-batch inputs [B][H][d] or [B][T][H][d]."""
        G, b, h0, NH = self.w.G, self.b, self.h0, self.nh
        hs, qs = slice(h0, h0 + NH), slice(h0 * G, (h0 + NH) * G)
        return tuple(np.ascontiguousarray(a[b:b + 1, ..., s, :]) for a, s in ((q, qs), (wq, hs), (wv, hs)))

    def cut_out(self, out_np):
        G = self.w.G
        return out_np[self.b:self.b + 1, ..., self.h0 * G:(self.h0 + self.nh) * G, :]

    def gpu_state(self, gpu):
        return to_np(gpu.values_view()[self.b:self.b + 1, self.h0:self.h0 + self.nh].contiguous(), self.w.dtype)


class LongRun:
    """The GPU trajectory of one workload and the oracles watching it; advance(t_end) moves it on."""

    def __init__(self, P, R, w, sample, replica, replica_steps, prompt_chunks, drift_every, nh=8):
        """sample, replica: (batch element, first KV head) of the nh memories each oracle holds (one oracle
        thread per memory)."""
        import torch
        self.P, self.R, self.w, self.torch = P, R, w, torch
        self.T = w.prefill_chunk if prompt_chunks else 0
        self.prompt = prompt_chunks * self.T
        self.total = w.decode_steps
        mk = syn.make_keys(w)
        self.mk = mk
        self.gpu = P.BctCache(w.M, w.B, w.Hq, w.Hkv, w.d, torch_dtype(w.dtype), w.scale, w.scale,
                              max_prefill_T=self.T)
        self.gpu.set_keys(to_dev(mk, w.dtype))
        self.nh = nh
        self.sample = Units(R, w, mk, *sample, nh)       # resynchronised on the GPU's state
        self.replica = Units(R, w, mk, *replica, nh)     # never sees the GPU's state
        self.replica_steps = replica_steps
        self.drift_every = drift_every
        rng = np.random.default_rng(syn.BASE_SEED + w.M)
        M = w.M
        self.samples = {M - 1, M, M + 1, 2 * M, self.total - 1} | {int(x) for x in rng.integers(64, self.total, 8)}
        self.samples = {t for t in self.samples if 64 <= t < self.total}
        self.t = 0
        self.gen = torch.Generator(device="cuda:0")
        self.gen.manual_seed(syn.BASE_SEED + 17 * w.M)
        self.block = None
        self.block_t0 = -(1 << 40)
        self.out = torch.empty((w.B, w.Hq, w.d), dtype=torch_dtype(w.dtype), device="cuda:0")
        self.worst_lock = self.worst_sample = self.worst_replica = 0.0
        self.done_samples = []

    # ---- the prompt
    def run_prompt(self):
        w, T = self.w, self.T
        for c in range(self.prompt // T):
            q, wq, wv = chunk_inputs(w, c * T, T)
            before = self.sample.gpu_state(self.gpu)
            o_gpu = to_np(self.gpu.prefill(to_dev(q, w.dtype), to_dev(wq, w.dtype), to_dev(wv, w.dtype), T), w.dtype)
            after = self.sample.gpu_state(self.gpu)
            sq, swq, swv = self.sample.cut(q, wq, wv)
            rq, rwq, rwv = self.replica.cut(q, wq, wv)
            assert all(np.array_equal(a, b) for a, b in zip((rq, rwq, rwv),
                                                            unit_inputs(w, c * T, self.replica.b, self.replica.h0, self.nh, T)))
            self.sample.ref.import_(None, before, c * T)
            with concurrent.futures.ThreadPoolExecutor(max_workers=3) as ex:   # three oracles, nh threads each
                f1 = ex.submit(self.sample.ref.prefill, sq, swq, swv, T)
                f2 = ex.submit(self.replica.ref.prefill, rq, rwq, rwv, T)
                f3 = ex.submit(prefill_mass, self.R, self.sample.ref, self.sample.mk, swq, T)
                o_ref, o_rep, mass = f1.result(), f2.result(), f3.result()
            what = f"{w.name} prompt chunk {c}"
            e = check_prefill_out(self.sample.cut_out(o_gpu), o_ref, w.dtype, what, max_ulp=8.0 if w.M > 8192 else 4.0)
            frac = check_prefill_state(self.R, self.sample.ref, self.sample.mk, swq, swv, after, T, what, mass=mass)
            er = float(np.max(np.abs(f64(self.replica.cut_out(o_gpu), w.dtype) - f64(o_rep, w.dtype))))
            assert er <= 2e-2, f"{what}: free-running replica out abs err {er:.3e}"
            self.worst_replica = max(self.worst_replica, er)
            assert np.array_equal(to_np(self.gpu.keys_view(), w.dtype), self.mk)
            _progress(f"{what} ({T} tokens): out within {e:.2f} ulp of the vector max, {frac:.3%} of the sampled "
                      f"state differs; replica out abs err {er:.2e}")
        assert self.gpu.steps == self.prompt

    # ---- decode
    def _device_block(self, t0):
        """Inputs of steps t0 .. t0+BLOCK-1 on the device; the replica's memories get bct_synth's values."""
        torch, w = self.torch, self.w
        dt = torch_dtype(w.dtype)
        blk = [torch.randn((BLOCK, w.B, H, w.d), generator=self.gen, device="cuda:0", dtype=torch.float32).to(dt)
               for H in (w.Hq, w.Hkv, w.Hkv)]
        n = min(BLOCK, self.replica_steps - t0)
        if n > 0:
            r, NH = self.replica, self.nh
            rows = [unit_inputs(w, self.prompt + t0 + i, r.b, r.h0, NH) for i in range(n)]
            for k, (lo, cnt) in enumerate(((r.h0 * w.G, NH * w.G), (r.h0, NH), (r.h0, NH))):
                host = np.concatenate([row[k] for row in rows], axis=0)        # [n][heads][d]
                blk[k][:n, r.b, lo:lo + cnt] = to_dev(host, w.dtype)
        self.block, self.block_t0 = blk, t0

    def _replica_step(self, t, o_gpu_dev):
        w, r, NH = self.w, self.replica, self.nh
        q, wq, wv = unit_inputs(w, self.prompt + t, r.b, r.h0, NH)
        o_rep = r.ref.decode_step(q, wq, wv)
        o_gpu = to_np(o_gpu_dev[r.b:r.b + 1, r.h0 * w.G:(r.h0 + NH) * w.G].contiguous(), w.dtype)
        g = f64(o_gpu, w.dtype)
        e = float(np.max(np.abs(g - f64(o_rep, w.dtype))))
        assert np.all(np.isfinite(g)) and e <= 2e-2, f"{w.name} step {t}: free-running replica out abs err {e:.3e}"
        self.worst_replica = max(self.worst_replica, e)
        if (t + 1) % self.drift_every == 0 or t + 1 == self.replica_steps:
            gs, rs = f64(r.gpu_state(self.gpu), w.dtype), f64(r.ref.values(), w.dtype)
            top = float(np.max(np.abs(rs)))
            drift = float(np.max(np.abs(gs - rs)) / bf16_ulp(top))
            _progress(f"{w.name}: replica after {self.prompt} prompt tokens + {t + 1} steps: state drift "
                      f"{drift:.2f} ulp of max|MV| = {top:.3g}, {np.mean(gs != rs):.3%} of elements differ, "
                      f"worst out abs err so far {self.worst_replica:.2e}")
            # every step can flip single roundings: a random walk of 1-ulp steps of the ELEMENT, far below this
            assert drift <= 32.0, f"{w.name}: replica state drift {drift:.1f} ulp"

    def advance(self, t_end):
        w, gpu, s = self.w, self.gpu, self.sample
        t_end = min(t_end, self.total)
        while self.t < t_end:
            t = self.t
            if t < 64 or t in self.samples:
                q, wq, wv = syn.make_step(w, self.prompt + t)
                if t == 0 or t >= 64:
                    before = s.gpu_state(gpu)
                    s.ref.import_(None, before, self.prompt + t)
                o_dev = gpu.decode_step(to_dev(q, w.dtype), to_dev(wq, w.dtype), to_dev(wv, w.dtype), self.out)
                o_ref = s.ref.decode_step(*s.cut(q, wq, wv))
                what = f"{w.name} step {t}"
                e = check_out(s.cut_out(to_np(o_dev, w.dtype)), o_ref, w.dtype, what)
                if t >= 64:
                    check_state_one_step(s.gpu_state(gpu), s.ref.values(), w.dtype, what, before=before)
                    assert np.array_equal(to_np(gpu.keys_view(), w.dtype), self.mk)
                    self.worst_sample = max(self.worst_sample, e)
                    self.done_samples.append(t)
                    _progress(f"{what}: resync ok, out abs err {e:.2e}")
                else:
                    self.worst_lock = max(self.worst_lock, e)
                    if t == 63:
                        _progress(f"{w.name}: 64 lock-step steps ok, worst out abs err {self.worst_lock:.2e}")
            else:
                if not (self.block_t0 <= t < self.block_t0 + BLOCK):
                    self._device_block(t - t % BLOCK)
                i = t - self.block_t0
                o_dev = gpu.decode_step(self.block[0][i], self.block[1][i], self.block[2][i], self.out)
            if t < self.replica_steps:
                self._replica_step(t, o_dev)
            self.t += 1
        if self.t == self.total:
            assert gpu.steps == self.prompt + self.total
            assert sorted(self.done_samples) == sorted(self.samples)
            assert self.torch.isfinite(gpu.values_view().float()).all()
            _progress(f"{w.name}: {self.prompt} prompt tokens + {self.total} decode steps done; worst out abs err: "
                      f"lock-step {self.worst_lock:.2e}, resync samples {self.worst_sample:.2e} "
                      f"(at steps {sorted(self.done_samples)}), free-running replica {self.worst_replica:.2e}")


# ------------------------------------------------------------------ cfg3

def test_cfg3_prompt_1024_then_8192_steps(P, R):
    w = syn.WORKLOADS["cfg3"]
    run = LongRun(P, R, w, sample=(31, 24), replica=(3, 0), replica_steps=w.decode_steps, prompt_chunks=2,
                  drift_every=1024)
    run.run_prompt()
    run.advance(w.decode_steps)


# ------------------------------------------------------------------ cfg4

def test_cfg4_gqa_16384_steps(P, R):
    w = syn.WORKLOADS["cfg4"]
    run = LongRun(P, R, w, sample=(63, 0), replica=(0, 0), replica_steps=1024, prompt_chunks=0, drift_every=256)
    run.advance(w.decode_steps)


# ------------------------------------------------------------------ cfg5, in segments (each well under two minutes)

@pytest.fixture(scope="module")
def cfg5_run(P, R):
    w = syn.WORKLOADS["cfg5"]
    return LongRun(P, R, w, sample=(7, 56), replica=(2, 8), replica_steps=1024, prompt_chunks=4, drift_every=256,
                   nh=4)


def test_cfg5_prompt_four_chunks_of_512(cfg5_run):
    cfg5_run.run_prompt()


@pytest.mark.parametrize("t_end", [2048, 16384, 32768, 49152, 65536])
def test_cfg5_decode_up_to(cfg5_run, t_end):
    assert cfg5_run.t == {2048: 0, 16384: 2048, 32768: 16384, 49152: 32768, 65536: 49152}[t_end], \
        "the segments of the cfg5 trajectory run in order"
    cfg5_run.advance(t_end)
