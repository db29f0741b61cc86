"""Host-only serving simulation over the library's allocator and scheduler (metadata-only arena):
how large a batch each reservation policy sustains and how many iterations a request pool takes.

Policies, as in the paper's evaluation (section 4, baselines): "max" reserves the maximum sequence
length for everybody (what a system must do that does not know the output length), "predicted"
reserves prompt + the upper edge of the predicted output-length bucket (10 buckets of max_len/10,
section 3; a wrong bucket with probability 1 - accuracy), "perfect" reserves the true total length.
A sequence that fills its reservation before it ends is doubled in place of eviction when room
exists, else evicted back to the pool with a doubled prediction (section 3, supervisor paragraph).
Lengths are synthetic (seeded); the paper's dataset is not available.
"""
import numpy as np

from . import binding as s3


def draw_requests(n, seed, max_len=2048):
    rng = np.random.default_rng(seed)
    prompt = rng.integers(8, 97, n)
    output = np.clip(np.rint(rng.lognormal(4.6, 0.9, n)), 1, max_len - 96).astype(np.int64)
    return prompt.astype(np.int64), output


def predicted_total(policy, prompt, output, max_len, seed, accuracy=0.9861, buckets=10):
    if policy == "max":
        return np.full_like(prompt, max_len)
    if policy == "perfect":
        return prompt + output
    rng = np.random.default_rng(seed + 1)
    width = -(-max_len // buckets)
    bucket = (output - 1) // width
    wrong = rng.random(prompt.size) > accuracy
    shift = np.where(rng.random(prompt.size) < 0.5, -1, 1)
    bucket = np.clip(np.where(wrong, bucket + shift, bucket), 0, buckets - 1)
    return np.minimum(max_len, prompt + (bucket + 1) * width)


def serve(policy, n_requests=4000, arena_bytes=68 * 10**9, n_layers=28, n_heads=16, head_dim=256, granule=64,
          max_len=2048, seed=0, n_kv_heads=0, kv_dtype=s3.S3_F16):
    """-> dict(avg_batch, iterations, grows, evictions, tokens).  One token per active sequence per
    iteration; the pool is offered to the scheduler at every iteration.  n_kv_heads / kv_dtype select
    the cache-footprint variants the paper's related-work section calls complementary (shared key/value
    heads, 8-bit rows): fewer bytes per token, so the same memory holds a larger batch."""
    cfg = s3.make_config(n_layers, n_heads, head_dim, kv_dtype, granule, max_len, n_kv_heads, s3.S3_F16)
    st, arena = s3.s3_kv_arena_init(cfg, None, arena_bytes)
    s3.check(st, "s3_kv_arena_init")
    st, sched = s3.s3_sched_create(arena)
    s3.check(st, "s3_sched_create")
    prompt, output = draw_requests(n_requests, seed, max_len)
    pred = predicted_total(policy, prompt, output, max_len, seed)
    total = prompt + output
    progress = prompt.copy()  # rows cached so far (kept across an eviction)
    for r in range(n_requests):
        s3.check(s3.s3_sched_submit(sched, r, int(pred[r])))
    act_req = np.zeros(0, np.int64)
    act_slot = np.zeros(0, np.int32)
    act_cap = np.zeros(0, np.int32)
    iterations = batch_sum = grows = evictions = 0
    done = 0
    while done < n_requests:
        rc, rid, sid, off, cap = s3.s3_sched_admit(sched, 1 << 16)
        s3.check(rc, "s3_sched_admit")
        if rc:
            act_req = np.concatenate([act_req, rid])
            act_slot = np.concatenate([act_slot, sid])
            act_cap = np.concatenate([act_cap, cap])
        if act_req.size == 0:
            raise RuntimeError("nothing fits the arena")
        # sequences whose reservation is full: double it, or go back to the pool with a doubled prediction
        keep = np.ones(act_req.size, bool)
        for i in np.nonzero(progress[act_req] >= act_cap)[0].tolist():
            st, new_off, new_cap = s3.s3_kv_grow(arena, int(act_slot[i]), int(act_cap[i]))
            if st == s3.S3_OK:
                act_cap[i] = new_cap
                grows += 1
            else:
                s3.check(s3.s3_kv_free(arena, int(act_slot[i])), "s3_kv_free")
                s3.check(s3.s3_sched_submit(sched, int(act_req[i]), int(min(max_len, 2 * act_cap[i]))))
                keep[i] = False
                evictions += 1
        act_req, act_slot, act_cap = act_req[keep], act_slot[keep], act_cap[keep]
        progress[act_req] += 1
        iterations += 1
        batch_sum += int(act_req.size)
        fin = progress[act_req] >= total[act_req]
        for slot in act_slot[fin].tolist():
            s3.check(s3.s3_kv_free(arena, slot), "s3_kv_free")
        done += int(fin.sum())
        act_req, act_slot, act_cap = act_req[~fin], act_slot[~fin], act_cap[~fin]
    s3.s3_sched_destroy(sched)
    s3.s3_kv_arena_destroy(arena)
    return dict(policy=policy, avg_batch=batch_sum / iterations, iterations=iterations, grows=grows,
                evictions=evictions, tokens=int(output.sum()), batch_sum=batch_sum)


if __name__ == "__main__":
    for pol in ("max", "predicted", "perfect"):
        print(serve(pol))
    print("8-bit rows:", serve("predicted", kv_dtype=s3.S3_E4M3))
    print("4 cached heads for 16 query heads:", serve("predicted", n_kv_heads=4))
