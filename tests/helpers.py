"""Shared test helpers: fixture parsing and small hand-built pools."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_kv(name):
    """Parse 'key = value' lines of a golden text file."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = line.split("=")
                out[k.strip()] = float(v)
    return out


def read_rows(name):
    """Parse whitespace-separated rows of a golden text file."""
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


ROUND_MODEL = dict(kv_bytes_per_token=1e5, flops_per_token=1e10, attn_flops_per_token2=1e6,
                   weight_bytes=1e10, nominal_batch=10.0)


def one_pool(F=1e13, B=1e12, backlog=2000, used=10000, cap=1000000, batch=100, qd=50,
             bw=1e9, lat=0.05):
    """1 prefill + 1 decode instance of one class."""
    pre = dict(flops=[F], hbm_bw=[B], backlog_tok=[backlog], type=[0])
    dec = dict(flops=[F], hbm_bw=[B], used_tok=[used], cap_tok=[cap], batch=[batch], qd_tok=[qd], type=[0])
    links = dict(n_types=1, bw=np.array([[bw]], np.float32),
                 latency=None if lat is None else np.array([[lat]], np.float32))
    return pre, dec, links


def random_pool(rng, P, D, T):
    """Small random heterogeneous pool with continuous rates (few ties)."""
    tF = rng.uniform(1e14, 3e15, T).astype(np.float32)
    tB = rng.uniform(5e11, 8e12, T).astype(np.float32)
    bw = rng.uniform(1e10, 1e11, (T, T)).astype(np.float32)
    lat = rng.uniform(0, 0.01, (T, T)).astype(np.float32)
    pt = rng.integers(0, T, P).astype(np.int32)
    dt = rng.integers(0, T, D).astype(np.int32)
    cap = rng.integers(50000, 400000, D).astype(np.int32)
    used = (rng.random(D) * cap).astype(np.int32)
    pre = dict(flops=tF[pt], hbm_bw=tB[pt], backlog_tok=rng.integers(0, 20001, P).astype(np.int32), type=pt)
    dec = dict(flops=tF[dt], hbm_bw=tB[dt], used_tok=used, cap_tok=cap,
               batch=np.clip(-(-used // 2048), 0, 256).astype(np.int32),
               qd_tok=rng.integers(0, 20001, D).astype(np.int32), type=dt)
    links = dict(n_types=T, bw=bw, latency=lat)
    types = dict(flops=tF, hbm_bw=tB)
    return types, pre, dec, links
