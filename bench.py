#!/usr/bin/env python3
"""Benchmark of the CFGzip hot path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W

Timed step = one decode step of the per-step path at batch 256, V = 128,256,
C = 8,000 (cfgzip_decode_step: fused expand + -inf apply with the token mask as
by-product and the map to representatives, one launch).  The same run also times the offline class build
(signatures + grouping) on the class-build workloads and the CPU oracle on a
bounded sample.  Prints ONE JSON line.

Logits rotate through several buffers whose total size exceeds the GPU's
memory-side cache, so every step streams its logits from HBM.
"""

from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E peak
N_LOGIT_BUFFERS = 8    # 8 x 65.7 MB = 525 MB > 256 MB memory-side cache
MASK_SOURCE = os.path.join(ROOT, "paper_2605_29986_amd", "csrc", "mask.hip")
MASK_COUNTERS = os.path.join(ROOT, "profiles", "mask_kernel_config5_hbm_counters.md")


def mask_kernel_traffic_bytes():
    """HBM bytes per launch of the mask kernel on this workload, as counted by rocprofv3 --pmc
    FETCH_SIZE and WRITE_SIZE (scaled by a plain copy of known size).  The summary of that
    measurement names the kernel source it was taken on by its SHA-256; if the source has changed
    since, the figure no longer describes the kernel and None is returned."""
    import hashlib
    import re
    try:
        text = open(MASK_COUNTERS).read()
        digest = hashlib.sha256(open(MASK_SOURCE, "rb").read()).hexdigest()
    except OSError:
        return None
    nbytes = re.search(r"^traffic_bytes_per_launch:\s*(\d+)", text, re.M)
    source = re.search(r"^kernel_source_sha256:\s*([0-9a-f]{64})", text, re.M)
    if not nbytes or not source or source.group(1) != digest:
        return None
    return int(nbytes.group(1))


def log(msg: str) -> None:
    print(msg, file=sys.stderr, flush=True)


def ensure_library():
    from paper_2605_29986_amd import binding, build
    if not os.path.exists(binding.library_path()):
        log("libcfgzip.so not found, building it with hipcc ...")
        build.build()
    return binding.load_library()


def event_ms(fn, stream):
    """Runs fn() between two HIP events recorded on `stream`; returns elapsed ms."""
    import torch
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    fn()
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1)


def decode_step_bytes(B: int, V: int, C: int) -> dict:
    Wv, Wc = (V + 31) // 32, (C + 31) // 32
    mask_kernel = 2 * B * V * 2 + B * Wv * 4 + B * Wc * 4 + V * 4
    map_kernel = B * 4 * 4
    return {"mask_kernel": mask_kernel, "step": mask_kernel + map_kernel}


def gather_ceiling(sizes):
    """Runs the calibration tool built next to the library: the rate of dependent 2-byte reads
    from an L2-resident [256][S] table by a kernel that does nothing else (best over 1, 2, 4, 8
    reads in flight per thread), per S and column pattern.  Returns {} if the tool is missing."""
    import subprocess
    from paper_2605_29986_amd import build
    if not os.path.exists(build.TOOL_PATH) or not sizes:
        return {}
    out = subprocess.run([build.TOOL_PATH] + [str(s) for s in sizes], capture_output=True, text=True,
                         timeout=120)
    best = {}
    for line in out.stdout.splitlines():
        try:
            rec = json.loads(line)
        except ValueError:
            continue
        key = (rec["S"], rec["column"])
        if key not in best or rec["reads_per_s"] > best[key]["reads_per_s"]:
            best[key] = rec
    return {f"S{S}_{col}": {"reads_per_s": rec["reads_per_s"], "in_flight": rec["in_flight"]}
            for (S, col), rec in best.items()}


def random_automaton(seed: int, S: int) -> np.ndarray:
    """Every transition drawn uniformly: no lexer structure at all (an input, seeded)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    table = rng.integers(0, S, size=(S, 256)).astype(np.uint16)
    table[0, :] = 0
    return table


def bench_class_build(lib_mod, raw, torch, configs, repeats: int, random_tables: bool = False):
    """Times cfgzip_signatures + cfgzip_build_classes on the class-build workloads.  With
    random_tables the vocabulary of each workload meets an automaton of the same size whose
    transitions are uniformly random: a byte then leaves about 0.63 S distinct states, the image
    walk saves nothing, the kept walk vectors overflow and the builder walks again to compare."""
    import synthetic_inputs as si
    out = {}
    stream = torch.cuda.current_stream()
    for idx in configs:
        cfg = si.make_config(idx)
        vocab, table = cfg["vocab"], cfg["table"]
        V, S = vocab.V, cfg["S"]
        if random_tables:
            table = random_automaton(cfg["seed"] + 4242, S)
        tb = torch.from_numpy(vocab.tok_bytes).cuda()
        to = torch.from_numpy(vocab.tok_off).cuda()
        tt = torch.from_numpy(table).cuda()
        stored = idx != 4 and not random_tables  # the largest workload hashes on the fly and verifies by re-walking
        sig = torch.empty((V, S), dtype=torch.uint16, device="cuda") if stored else None
        h = torch.empty((V,), dtype=torch.int64, device="cuda")
        c = torch.empty((V,), dtype=torch.int32, device="cuda")
        r = torch.empty((V,), dtype=torch.int32, device="cuda")
        ws_sig = torch.empty(raw.cfgzip_signatures_workspace_bytes(V, S), dtype=torch.uint8, device="cuda")
        ws_bld = torch.empty(raw.cfgzip_build_classes_workspace_bytes(V, S), dtype=torch.uint8, device="cuda")
        res = {}

        def run_sig():
            lib_mod.cfgzip_signatures(tb, to, tt, want_sig=stored, sig_out=sig, hash_out=h,
                                      workspace=ws_sig)

        def run_build():
            res["out"] = lib_mod.cfgzip_build_classes(tb, to, tt, sig, h, class_of_token=c,
                                                      rep_of_class=r, workspace=ws_bld,
                                                      signatures_workspace=ws_sig)

        # the same signatures by composition over token prefixes (Appendix A, Lemma 1)
        ws_cmp = torch.empty(raw.cfgzip_signatures_composed_workspace_bytes(V, S), dtype=torch.uint8, device="cuda")

        def run_sig_composed():
            lib_mod.cfgzip_signatures(tb, to, tt, want_sig=stored, sig_out=sig, hash_out=h,
                                      workspace=ws_cmp, composed=True)

        run_sig_composed(); run_sig(); run_build(); torch.cuda.synchronize()  # warm-up
        t_sig, t_all, t_cmp = [], [], []
        for _ in range(repeats):
            t_cmp.append(event_ms(run_sig_composed, stream))
            t_sig.append(event_ms(run_sig, stream))
            t_all.append(event_ms(lambda: (run_sig(), run_build()), stream))
        C, collisions = res["out"][2], res["out"][3]
        sum_len = int(vocab.tok_off[-1])
        ms_sig, ms_all = min(t_sig), min(t_all)
        # table reads: a plain walk from every state does S reads per token byte; the image walk
        # does one read per distinct state of the first byte's column and remaining byte
        # (input statistics only, computed here for the report)
        nimg = np.array([np.unique(table[:, b]).size for b in range(256)] + [S], dtype=np.int64)
        lens = np.diff(vocab.tok_off)
        first = np.where(lens > 0, vocab.tok_bytes[np.minimum(vocab.tok_off[:-1], max(sum_len - 1, 0))], 256)
        reads_done = int((nimg[first] * np.maximum(lens - 1, 0)).sum())
        kept = bool((nimg[first] <= min(S, 256)).all())
        # table reads left when every token of four bytes or more starts from its longest prefix
        # of two or three bytes that is itself a token (input statistics, for the report)
        short = {bytes(vocab.token(t)) for t in np.nonzero((lens >= 2) & (lens <= 3))[0]}
        reads_composed = 0
        for t in range(V):
            L = int(lens[t])
            if L == 0:
                continue
            skip = 1
            if L > 3:
                tok = bytes(vocab.token(t))
                skip = 3 if tok[:3] in short else (2 if tok[:2] in short else 1)
            reads_composed += int(nimg[first[t]]) * (L - skip)
        entry = {
            "V": V, "S": S, "C": C, "V_over_C": round(V / C, 2), "sig_stored": stored,
            "automaton": "uniformly random transitions" if random_tables else "lexer-like (synthetic_inputs)",
            "ms_signatures": round(ms_sig, 4), "ms_build_total": round(ms_all, 4),
            "ms_signatures_by_composition": round(min(t_cmp), 4),
            "table_reads_by_composition": reads_composed,
            "ms_grouping": round(ms_all - ms_sig, 4),
            # EFFECTIVE rates: V * S token-state pairs get their end state per call, but the image
            # walk does not perform V * S walks: it reads table_reads_image_walk table entries
            # where a plain walk reads table_reads_plain_walk
            "walks_per_s": V * S / (ms_all * 1e-3),
            "walks_per_s_signatures_only": V * S / (ms_sig * 1e-3),
            "walks_per_s_kind": "effective (token-state pairs resolved per second)",
            "table_reads_plain_walk": S * sum_len,
            "table_reads_image_walk": reads_done,
            "table_reads_ratio": round(reads_done / max(S * sum_len, 1), 4),
            "mean_image_states_per_token": round(float(nimg[first].mean()), 1),
            "walk_vectors_kept_for_the_builder": kept,
            "comparison_source": "kept walk vectors" if kept else "second walk (the kept vectors overflowed)",
            "collisions": collisions,
            "sig_store_GBps": round(2 * V * S / (ms_sig * 1e-3) / 1e9, 1) if stored else None,
            # table reads of the image walk per second over the whole call (tables included)
            "table_reads_per_s": reads_done / (ms_sig * 1e-3),
        }
        out[f"config{idx}"] = entry
        log(f"class build config {idx}{' (random automaton)' if random_tables else ''}: V={V} S={S} C={C} "
            f"signatures {ms_sig:.3f} ms, total {ms_all:.3f} ms, {V * S / (ms_all * 1e-3):.3e} effective walks/s "
            f"({reads_done:.3e} of {S * sum_len:.3e} table reads done)")
        log(f"  signatures by composition over token prefixes: {min(t_cmp):.3f} ms "
            f"({reads_composed:.3e} table reads)")
        del sig, h, c, r, ws_sig, ws_bld, ws_cmp
    return out


def bench_displacement(lib_mod, raw, torch, repeats: int, cpu_sample: int, grammar: str = "json"):
    """General case: displacement sets of config 3's vocabulary over a grammar in Greibach normal
    form (the JSON value language, or the C-flavoured statement language), then the classes from
    the rows.  cpu_sample > 0 also times the oracle (pure Python, one core) on that many leading
    tokens."""
    import synthetic_inputs as si
    from synthetic_inputs.grammar import make_clike_gnf, make_json_gnf
    g = make_json_gnf() if grammar == "json" else make_clike_gnf()
    name = "JSON grammar" if grammar == "json" else "C-flavoured statement grammar"
    vocab = si.make_config(3)["vocab"]
    V = vocab.V
    stream = torch.cuda.current_stream()
    tb = torch.from_numpy(vocab.tok_bytes).cuda()
    to = torch.from_numpy(vocab.tok_off).cuda()
    gd = [torch.from_numpy(x).cuda() for x in g.arrays()]
    ws = torch.empty(raw.cfgzip_displacements_workspace_bytes(V, g.N, g.P), dtype=torch.uint8, device="cuda")
    # rows long enough for every set of these workloads (no token left in a class of its own for
    # want of room); the shortest row length is timed beside it
    ROW = 1024
    ws_bld = torch.empty(raw.cfgzip_build_classes_workspace_bytes(V, ROW), dtype=torch.uint8,
                         device="cuda")
    c = torch.empty((V,), dtype=torch.int32, device="cuda")
    r = torch.empty((V,), dtype=torch.int32, device="cuda")
    res = {}

    def run_adj():
        lib_mod.cfgzip_stack_adjacency(*gd, g.N, workspace=ws)

    def run_disp():
        res["rows"] = lib_mod.cfgzip_displacements(tb, to, *gd, g.N, row_len=ROW, workspace=ws)

    def run_build():
        rows, hashes, _st = res["rows"]
        res["cls"] = lib_mod.cfgzip_build_classes(tb, to, None, rows, hashes, class_of_token=c,
                                                  rep_of_class=r, workspace=ws_bld)

    run_adj(); run_disp(); run_build(); torch.cuda.synchronize()
    t_adj, t_disp, t_all = [], [], []
    for _ in range(repeats):
        t_adj.append(event_ms(run_adj, stream))
        t_disp.append(event_ms(run_disp, stream))
        t_all.append(event_ms(lambda: (run_disp(), run_build()), stream))
    status = res["rows"][2].cpu().numpy()
    C = res["cls"][2]
    ms_all = min(t_all)
    out = {
        "workload": "%s in Greibach normal form (%d non-terminals, %d productions) x "
                    "config 3 vocabulary" % (name, g.N, g.P),
        "V": V, "N": g.N, "P": g.P, "C": C, "V_over_C": round(V / C, 2), "row_len": ROW,
        "overflow_tokens": int((status == lib_mod.DISP_OVERFLOW).sum()),
        "ms_stack_adjacency": round(min(t_adj), 4),
        "ms_displacements": round(min(t_disp), 4),     # adjacency included
        "ms_total_with_classes": round(ms_all, 4),
        "tokens_per_s": V / (ms_all * 1e-3),
        "token_bytes_per_s": int(vocab.tok_off[-1]) / (min(t_disp) * 1e-3),
    }
    log(f"displacement ({name}): V={V} N={g.N} P={g.P} C={C} overflow={out['overflow_tokens']} adjacency "
        f"{min(t_adj):.3f} ms, displacements {min(t_disp):.3f} ms, with classes {ms_all:.3f} ms")
    # the same with the shortest rows the library takes: sets that need more become singletons
    ws_bld4 = torch.empty(raw.cfgzip_build_classes_workspace_bytes(V, 256), dtype=torch.uint8, device="cuda")

    def run_short():
        rows, hashes, st = lib_mod.cfgzip_displacements(tb, to, *gd, g.N, row_len=256, workspace=ws)
        res["short"] = (lib_mod.cfgzip_build_classes(tb, to, None, rows, hashes, class_of_token=c,
                                                     rep_of_class=r, workspace=ws_bld4), st)

    run_short(); torch.cuda.synchronize()
    ms_short = min(event_ms(run_short, stream) for _ in range(repeats))
    out["row_len_256"] = {"C": res["short"][0][2], "ms_total_with_classes": round(ms_short, 4),
                          "overflow_tokens": int((res["short"][1].cpu().numpy() == lib_mod.DISP_OVERFLOW).sum())}
    log(f"displacement, 256-entry rows: C={out['row_len_256']['C']} overflow="
        f"{out['row_len_256']['overflow_tokens']} with classes {ms_short:.3f} ms")
    if cpu_sample > 0:
        from oracle import displacement as D
        import oracle
        n = min(cpu_sample, V)
        toks = vocab.tokens()[:n]
        prods = g.productions()
        t0 = time.perf_counter()
        rows, _h, _st = D.displacement_rows(toks, prods, seed=1, row_len=ROW)
        oracle.build_classes(rows, vocab.tok_off[:n + 1])
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": n / dt, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                               "sample": f"first {n} tokens of the same vocabulary, same grammar "
                                         "(adjacency, bounded Algorithm 1, row encoding, grouping)"}
    return out


def bench_nfa(lib_mod, raw, torch, repeats: int, cpu: bool):
    """Non-deterministic lexer: config 2's vocabulary against its automaton with a tenth of the
    live transitions doubled; relations, then classes from the relation rows."""
    import synthetic_inputs as si
    from synthetic_inputs.nfa import make_lexer_nfa
    cfg = si.make_config(2)
    vocab, S = cfg["vocab"], cfg["S"]
    nfa_np = make_lexer_nfa(cfg["seed"] + 500, S, 0.10)
    V, W = vocab.V, nfa_np.shape[2]
    stream = torch.cuda.current_stream()
    tb = torch.from_numpy(vocab.tok_bytes).cuda()
    to = torch.from_numpy(vocab.tok_off).cuda()
    nfa = torch.from_numpy(nfa_np.view(np.int32)).cuda()
    row_len = 2 * S * W
    ws_bld = torch.empty(raw.cfgzip_build_classes_workspace_bytes(V, row_len), dtype=torch.uint8, device="cuda")
    c = torch.empty((V,), dtype=torch.int32, device="cuda")
    r = torch.empty((V,), dtype=torch.int32, device="cuda")
    res = {}

    def run_rel():
        res["rel"] = lib_mod.cfgzip_nfa_signatures(tb, to, nfa)

    def run_build():
        rel, h = res["rel"]
        res["cls"] = lib_mod.cfgzip_build_classes(tb, to, None, rel.view(torch.uint16).reshape(V, row_len), h,
                                                  class_of_token=c, rep_of_class=r, workspace=ws_bld)

    run_rel(); run_build(); torch.cuda.synchronize()
    t_rel, t_all = [], []
    for _ in range(repeats):
        t_rel.append(event_ms(run_rel, stream))
        t_all.append(event_ms(lambda: (run_rel(), run_build()), stream))
    ms_rel, ms_all = min(t_rel), min(t_all)
    C = res["cls"][2]
    out = {
        "workload": "config 2 vocabulary x its 256-state lexer with 10 % of the live transitions doubled",
        "V": V, "S": S, "C": C, "V_over_C": round(V / C, 2),
        "ms_relations": round(ms_rel, 4), "ms_total_with_classes": round(ms_all, 4),
        "walks_per_s": V * S / (ms_all * 1e-3),
        "relation_store_GBps": round(V * S * W * 4 / (ms_rel * 1e-3) / 1e9, 1),
    }
    log(f"nfa: V={V} S={S} C={C} relations {ms_rel:.3f} ms ({out['relation_store_GBps']} GB/s stored), "
        f"with classes {ms_all:.3f} ms, {out['walks_per_s']:.3e} walks/s")
    # engine side over state sets: per-state class masks once, then per step the class masks of
    # 256 state sets and their advance on the representatives of sampled tokens
    rel_t, _h = res["rel"]
    c_t, r_t = res["cls"][0], res["cls"][1]
    rel_rep = rel_t[r_t.long()].contiguous()          # plumbing: rows of the representatives
    rng = np.random.Generator(np.random.PCG64(cfg["seed"] + 600))
    live = torch.from_numpy((rng.random(S) < 0.5).astype(np.uint8)).cuda()
    state_mask = lib_mod.cfgzip_nfa_state_masks(rel_rep, live)
    ms_sm = min(event_ms(lambda: lib_mod.cfgzip_nfa_state_masks(rel_rep, live), stream) for _ in range(repeats))
    Bn = 256
    members = np.zeros((Bn, W * 32), bool)
    for b in range(Bn):
        members[b, rng.integers(1, S, size=2)] = True
    sets0 = torch.from_numpy(np.packbits(members, axis=1, bitorder="little").view(np.int32)).cuda()
    tok_t = torch.from_numpy(rng.integers(0, V, size=Bn).astype(np.int32)).cuda()
    sets = sets0.clone()

    def engine_steps(n=100):
        for _ in range(n):
            lib_mod.cfgzip_nfa_class_masks(state_mask, C, sets)
            lib_mod.cfgzip_nfa_advance_states(rel_rep, c_t, tok_t, sets)
    engine_steps(5)
    us_step = event_ms(engine_steps, stream) * 1e3 / 100
    out["engine_over_state_sets"] = {"B": Bn, "ms_state_masks_once": round(ms_sm, 4),
                                     "us_per_step_class_masks_plus_advance": round(us_step, 2)}
    log(f"nfa engine: state masks [S={S}][C={C}] once {ms_sm * 1e3:.1f} us; class masks + advance of {Bn} state sets "
        f"{us_step:.1f} us per step")
    if cpu:
        import oracle
        t0 = time.perf_counter()
        rel = oracle.nfa_signatures(vocab.tok_bytes, vocab.tok_off, nfa_np)
        oracle.build_classes(np.ascontiguousarray(rel).view(np.uint16).reshape(V, row_len), vocab.tok_off)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": V * S / dt, "unit": "walks/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": "the whole workload"}
    return out


def cpu_baseline_decode(c5, r5, d, budget_s: float = 10.0, max_steps: int = 2000):
    """The oracle's decode step (expand, apply, map) on full-size steps, timed on the host."""
    import oracle
    B, V, C = d["B"], d["V"], d["C"]
    logits = d["logits"].copy()
    lib = oracle._load()
    tok_bits = np.empty((B, (V + 31) // 32), dtype=np.int32)
    out = np.empty(B, dtype=np.int32)
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    steps, t0 = 0, time.perf_counter()
    while steps < max_steps and (steps == 0 or time.perf_counter() - t0 < budget_s):
        lib.oracle_expand_mask(p(d["cls_bits"]), ctypes.c_int32(B), ctypes.c_int32(C), p(c5),
                               ctypes.c_int32(V), p(tok_bits))
        lib.oracle_apply_mask_bf16(p(logits), ctypes.c_int32(B), ctypes.c_int32(V),
                                   ctypes.c_int64(V), p(tok_bits))
        lib.oracle_map_to_rep(p(d["tok"]), ctypes.c_int32(B), p(c5), ctypes.c_int32(V), p(r5),
                              ctypes.c_int32(C), p(out))
        steps += 1
    dt = time.perf_counter() - t0
    nbytes = decode_step_bytes(B, V, C)["step"]
    return {"value": nbytes * steps / dt / 1e9, "unit": "GB/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"{steps} full-size decode steps (B={B}, V={V}, C={C}) in {dt:.2f} s, "
                      f"OpenMP over batch rows"}


def cpu_baseline_build(idx: int, random_table: bool = False):
    import oracle
    import synthetic_inputs as si
    cfg = si.make_config(idx)
    vocab, table = cfg["vocab"], cfg["table"]
    if random_table:
        table = random_automaton(cfg["seed"] + 4242, cfg["S"])
    t0 = time.perf_counter()
    sig = oracle.signatures(vocab.tok_bytes, vocab.tok_off, table)
    t1 = time.perf_counter()
    oracle.build_classes(sig, vocab.tok_off)
    t2 = time.perf_counter()
    return {"workload": f"config {idx}", "walks_per_s": vocab.V * cfg["S"] / (t2 - t0),
            "s_signatures": round(t1 - t0, 4), "s_grouping": round(t2 - t1, 4),
            "cores": oracle.num_threads(), "kind": "oracle"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--p-allowed", type=float, default=0.5)
    ap.add_argument("--build-configs", type=str, default="2,3,4")
    ap.add_argument("--build-repeats", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-random-automata", action="store_true",
                    help="skip the class build against uniformly random automata")
    ap.add_argument("--no-displacement", action="store_true",
                    help="skip the grammar and non-deterministic automaton pre-computation workloads")
    ap.add_argument("--mask-variants", action="store_true",
                    help="also time the other forms of the mask path at the same shape")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on exactly one GPU (the path has no cross-GPU part); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the CFGzip path has no CPU fallback", file=sys.stderr)
        return 3
    raw = ensure_library()
    import paper_2605_29986_amd as lib_mod
    import synthetic_inputs as si

    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    sptr = ctypes.c_void_p(int(stream.cuda_stream))

    # ---- class map of the decode workload: config-3 class build on the GPU, resized to C = 8000
    B, C = 256, 8000
    cfg = si.make_config(5)
    vocab, table = cfg["vocab"], cfg["table"]
    V = vocab.V
    tb = torch.from_numpy(vocab.tok_bytes).cuda()
    to = torch.from_numpy(vocab.tok_off).cuda()
    tt = torch.from_numpy(table).cuda()
    sig, h = lib_mod.cfgzip_signatures(tb, to, tt)
    c3, r3, C3, _ = lib_mod.cfgzip_build_classes(tb, to, tt, sig, h)
    c5_np, r5_np = si.adjust_class_count(c3.cpu().numpy(), C)
    del sig, h
    log(f"decode workload: V={V}, config-3 build gave C={C3}, resized to C={C}")

    d = si.make_decode_inputs(si.config_seed(5), B, V, C, "bf16", p_allowed=args.p_allowed, sigma=2.0)
    c5 = torch.from_numpy(c5_np).cuda()
    r5 = torch.from_numpy(r5_np).cuda()
    logits0 = torch.from_numpy(d["logits"]).cuda().view(torch.bfloat16)
    logit_bufs = [logits0] + [logits0.clone() for _ in range(N_LOGIT_BUFFERS - 1)]
    rng = np.random.Generator(np.random.PCG64(si.config_seed(5) + 77))
    cls_bufs = [torch.from_numpy(d["cls_bits"]).cuda()]
    for _ in range(N_LOGIT_BUFFERS - 1):
        words = rng.integers(0, 2 ** 32, size=d["cls_bits"].shape, dtype=np.uint64).astype(np.uint32)
        if args.p_allowed != 0.5:
            bits = rng.random((B, d["cls_bits"].shape[1] * 32)) < args.p_allowed
            words = np.packbits(bits, axis=1, bitorder="little").view(np.uint32).reshape(B, -1)
        cls_bufs.append(torch.from_numpy(words.view(np.int32)).cuda())
    tok = torch.from_numpy(d["tok"]).cuda()
    tok_bits = torch.empty((B, (V + 31) // 32), dtype=torch.int32, device="cuda")
    rep_out = torch.empty((B,), dtype=torch.int32, device="cuda")

    i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
    mask_args = [(vp(lb.data_ptr()), i32(1), i32(B), i32(V), i64(V), vp(cb.data_ptr()), i32(1),
                  vp(c5.data_ptr()), i32(C), vp(tok_bits.data_ptr()), sptr)
                 for lb, cb in zip(logit_bufs, cls_bufs)]
    map_args = (vp(tok.data_ptr()), i32(B), vp(c5.data_ptr()), i32(V), vp(r5.data_ptr()), i32(C),
                vp(rep_out.data_ptr()), sptr)
    apply_mask, map_to_rep = raw.cfgzip_apply_mask, raw.cfgzip_map_to_rep
    # the timed step: mask and map in one launch (cfgzip_decode_step)
    step_args = [(vp(lb.data_ptr()), i32(1), i32(B), i32(V), i64(V), vp(cb.data_ptr()), vp(c5.data_ptr()),
                  i32(C), vp(tok_bits.data_ptr()), vp(tok.data_ptr()), vp(r5.data_ptr()),
                  vp(rep_out.data_ptr()), sptr) for lb, cb in zip(logit_bufs, cls_bufs)]
    decode_step = raw.cfgzip_decode_step

    def step(i: int) -> None:
        rc = decode_step(*step_args[i % N_LOGIT_BUFFERS])
        if rc != 0:
            raise RuntimeError(f"decode step failed, rc={rc}")

    def step_two_calls(i: int) -> None:
        rc = apply_mask(*mask_args[i % N_LOGIT_BUFFERS])
        rc |= map_to_rep(*map_args)
        if rc != 0:
            raise RuntimeError(f"decode step failed, rc={rc}")

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = wall_ms / args.steps
    # the same step as two calls (cfgzip_apply_mask, then cfgzip_map_to_rep): context
    for i in range(args.warmup):
        step_two_calls(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step_two_calls(i)
    torch.cuda.synchronize()
    ms_per_step_two_calls = (time.perf_counter() - t0) * 1e3 / args.steps

    # dominant kernel alone, HIP events on its stream
    def mask_only():
        for i in range(args.steps):
            apply_mask(*mask_args[i % N_LOGIT_BUFFERS])
    mask_ms = event_ms(mask_only, stream) / args.steps
    # same kernel on one buffer only (logits resident in the memory-side cache): context
    def mask_one_buffer():
        for _ in range(args.steps):
            apply_mask(*mask_args[0])
    mask_cached_ms = event_ms(mask_one_buffer, stream) / args.steps

    # a plain device-to-device copy of one logits buffer (known size: read 65.7 MB, write 65.7 MB);
    # profiler byte counters are calibrated against it
    calib = torch.empty_like(logits0)
    for _ in range(5):
        calib.copy_(logits0)
    torch.cuda.synchronize()
    del calib

    nbytes = decode_step_bytes(B, V, C)
    value = nbytes["step"] / (ms_per_step * 1e-3) / 1e9
    achieved = nbytes["mask_kernel"] / (mask_ms * 1e-3) / 1e9
    log(f"decode step: {ms_per_step * 1e3:.2f} us/step -> {value:.1f} GB/s; mask kernel alone "
        f"{mask_ms * 1e3:.2f} us -> {achieved:.1f} GB/s ({achieved / HBM_PEAK_GBS:.1%} of HBM peak); "
        f"one-buffer (cache-resident) {mask_cached_ms * 1e3:.2f} us")

    # ---- engine side for the byte automaton (next row after the hot path): per-state class
    # masks once, then a closed step = class masks from states, fused expand + apply, advance on
    # the representatives of the sampled tokens
    rep_tokens = [vocab.token(int(t)) for t in r5_np]
    rep_off = np.zeros(C + 1, dtype=np.int64)
    rep_off[1:] = np.cumsum([len(t) for t in rep_tokens])
    rep_bytes = np.frombuffer(b"".join(rep_tokens), dtype=np.uint8).copy()
    sig_rep, _ = lib_mod.cfgzip_signatures(torch.from_numpy(rep_bytes).cuda(),
                                           torch.from_numpy(rep_off).cuda(), tt, want_hash=False)
    S5 = int(table.shape[0])
    live_np = (rng.random(S5) < 0.5).astype(np.uint8)
    live_np[0] = 0
    live = torch.from_numpy(live_np).cuda()
    state_mask = torch.empty((S5, (C + 31) // 32), dtype=torch.int32, device="cuda")
    lib_mod.cfgzip_state_masks(sig_rep, live, state_mask=state_mask)
    ms_state_masks = min(event_ms(lambda: lib_mod.cfgzip_state_masks(sig_rep, live, state_mask=state_mask),
                                  stream) for _ in range(5))
    states = torch.from_numpy(rng.integers(1, S5, size=B).astype(np.int32)).cuda()
    cls_engine = torch.empty((B, (C + 31) // 32), dtype=torch.int32, device="cuda")
    cm_args = (vp(state_mask.data_ptr()), i32(S5), i32(C), vp(states.data_ptr()), i32(B),
               vp(cls_engine.data_ptr()), sptr)
    adv_args = (vp(sig_rep.data_ptr()), i32(C), i32(S5), vp(c5.data_ptr()), i32(V), vp(tok.data_ptr()),
                i32(B), vp(states.data_ptr()), sptr)
    eng_mask_args = [(vp(lb.data_ptr()), i32(1), i32(B), i32(V), i64(V), vp(cls_engine.data_ptr()), i32(1),
                      vp(c5.data_ptr()), i32(C), vp(tok_bits.data_ptr()), sptr) for lb in logit_bufs]

    def engine_steps():
        for i in range(args.steps):
            rc = raw.cfgzip_class_masks(*cm_args)
            rc |= apply_mask(*eng_mask_args[i % N_LOGIT_BUFFERS])
            rc |= raw.cfgzip_advance_states(*adv_args)
            if rc != 0:
                raise RuntimeError(f"engine step failed, rc={rc}")
    engine_steps()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    engine_steps()
    torch.cuda.synchronize()
    engine_us = (time.perf_counter() - t0) * 1e6 / args.steps
    # the same step in one launch: states alternate between two arrays
    states2 = [states, torch.empty_like(states)]
    one_args = [(vp(lb.data_ptr()), i32(1), i32(B), i32(V), i64(V), vp(state_mask.data_ptr()), i32(S5), i32(C),
                 vp(c5.data_ptr()), vp(sig_rep.data_ptr()), vp(tok.data_ptr()), vp(states2[i % 2].data_ptr()),
                 vp(states2[(i + 1) % 2].data_ptr()), vp(tok_bits.data_ptr()), sptr)
                for i, lb in enumerate(logit_bufs)]

    def engine_steps_one_launch():
        for i in range(args.steps):
            rc = raw.cfgzip_engine_step(*one_args[i % N_LOGIT_BUFFERS])
            if rc != 0:
                raise RuntimeError(f"engine step failed, rc={rc}")
    engine_steps_one_launch()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    engine_steps_one_launch()
    torch.cuda.synchronize()
    engine_one_us = (time.perf_counter() - t0) * 1e6 / args.steps
    engine = {"workload": f"closed step: class masks from {B} automaton states (S={S5}, C={C}), fused "
                          "expand + apply on bf16 logits, state advance on representatives",
              "us_per_step": round(engine_us, 2),
              "GBps": round(nbytes["mask_kernel"] / (engine_us * 1e-6) / 1e9, 1),
              "us_per_step_one_launch": round(engine_one_us, 2),
              "GBps_one_launch": round(nbytes["mask_kernel"] / (engine_one_us * 1e-6) / 1e9, 1),
              "ms_state_masks_once": round(ms_state_masks, 4)}
    log(f"engine step (class masks + fused mask + advance): {engine_us:.2f} us/step, in one launch "
        f"{engine_one_us:.2f} us/step; state masks [S={S5}][C={C}] once: {ms_state_masks * 1e3:.1f} us")

    # ---- optional: the other forms of the mask path at the same shape (kernel alone, rotating buffers)
    mask_variants = {}
    if args.mask_variants:
        def time_loop(call_args_list, fn):
            def loop():
                for i in range(args.steps):
                    fn(*call_args_list[i % len(call_args_list)])
            loop()
            return event_ms(loop, stream) / args.steps * 1e3  # us per launch
        bf16_rw = 2 * B * V * 2
        bits_v, bits_c, ids = B * ((V + 31) // 32) * 4, B * ((C + 31) // 32) * 4, V * 4
        us = time_loop([a[:9] + (None,) + a[10:] for a in mask_args], apply_mask)
        mask_variants["bf16_fused_no_token_mask_out"] = {"us": round(us, 2), "GBps": round((bf16_rw + bits_c + ids) / us / 1e3, 1)}
        us = time_loop([(vp(cb.data_ptr()), i32(B), i32(C), vp(c5.data_ptr()), i32(V), vp(tok_bits.data_ptr()), sptr)
                        for cb in cls_bufs], raw.cfgzip_expand_mask)
        mask_variants["expand_only"] = {"us": round(us, 2), "GBps": round((bits_v + bits_c + ids) / us / 1e3, 1)}
        us = time_loop([(vp(lb.data_ptr()), i32(1), i32(B), i32(V), i64(V), vp(tok_bits.data_ptr()), i32(0),
                         None, i32(0), None, sptr) for lb in logit_bufs], apply_mask)
        mask_variants["bf16_apply_from_token_mask"] = {"us": round(us, 2), "GBps": round((bf16_rw + bits_v) / us / 1e3, 1)}
        f32_bufs = [torch.randn((B, V), dtype=torch.float32, device="cuda") for _ in range(4)]
        us = time_loop([(vp(fb.data_ptr()), i32(0), i32(B), i32(V), i64(V), vp(cls_bufs[0].data_ptr()), i32(1),
                         vp(c5.data_ptr()), i32(C), vp(tok_bits.data_ptr()), sptr) for fb in f32_bufs], apply_mask)
        mask_variants["f32_fused_token_mask_out"] = {"us": round(us, 2),
                                                     "GBps": round((2 * B * V * 4 + bits_v + bits_c + ids) / us / 1e3, 1)}
        del f32_bufs
        for k, v in mask_variants.items():
            log(f"mask variant {k}: {v['us']} us -> {v['GBps']} GB/s")

    build_cfgs = [int(x) for x in args.build_configs.split(",") if x]
    class_build = bench_class_build(lib_mod, raw, torch, build_cfgs, args.build_repeats) if build_cfgs else {}
    # ceiling for the walk's table reads when the table is read from L2 (S > 256): measured, same run
    ceilings = gather_ceiling(sorted({v["S"] for v in class_build.values() if v["S"] > 256}))
    for v in class_build.values():
        c = ceilings.get(f"S{v['S']}_wave-uniform")
        if c:
            v["table_read_ceiling_per_s"] = c["reads_per_s"]
            v["frac_of_table_read_ceiling"] = round(v["table_reads_per_s"] / c["reads_per_s"], 4)
            log(f"S={v['S']}: {v['table_reads_per_s']:.3e} table reads/s in the signature call, "
                f"pure-gather ceiling {c['reads_per_s']:.3e} ({v['frac_of_table_read_ceiling']:.1%})")
    # the same vocabularies against automata without any structure (the image walk's worst case)
    class_build_random = {}
    if build_cfgs and not args.no_random_automata:
        class_build_random = bench_class_build(lib_mod, raw, torch, [i for i in build_cfgs if i in (3, 4)],
                                               args.build_repeats, random_tables=True)
        for v in class_build_random.values():
            c = ceilings.get(f"S{v['S']}_wave-uniform")
            if c:
                v["table_read_ceiling_per_s"] = c["reads_per_s"]
                v["frac_of_table_read_ceiling"] = round(v["table_reads_per_s"] / c["reads_per_s"], 4)
                log(f"random automaton S={v['S']}: {v['table_reads_per_s']:.3e} table reads/s in the signature "
                    f"call, pure-gather ceiling {c['reads_per_s']:.3e} ({v['frac_of_table_read_ceiling']:.1%})")
    if ceilings:
        class_build["gather_ceiling"] = ceilings

    result = {
        "metric": "masked-logits GB/s per decode step (class mask -> token mask, -inf apply, "
                  "map to representative); class build in token-state walks/s under class_build",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "config 5: decode step, batch 256, V=128256, C=8000, bf16 logits "
                               "N(0, sigma=2), class masks Bernoulli(%g), %d rotating logit buffers"
                               % (args.p_allowed, N_LOGIT_BUFFERS),
                   "B": B, "V": V, "C": C, "bytes_per_step": nbytes["step"]},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": mask_kernel_traffic_bytes(),
                     "kernel": "mask_kernel<bf16, class bits, token bits out, 16-byte accesses>",
                     "bytes_per_launch": nbytes["mask_kernel"],
                     "us_per_launch": round(mask_ms * 1e3, 3),
                     "us_per_launch_cache_resident": round(mask_cached_ms * 1e3, 3)},
        "ms_per_step_two_calls": round(ms_per_step_two_calls, 6),
        "class_build": class_build,
        "class_build_random_automaton": class_build_random,
        "engine": engine,
    }
    if not args.no_displacement:
        result["nfa"] = bench_nfa(lib_mod, raw, torch, args.build_repeats, not args.no_cpu_baseline)
        result["displacement"] = bench_displacement(lib_mod, raw, torch, args.build_repeats,
                                                    0 if args.no_cpu_baseline else 30000)
        result["displacement_clike"] = bench_displacement(lib_mod, raw, torch, args.build_repeats,
                                                          0 if args.no_cpu_baseline else 30000, "clike")
    if mask_variants:
        result["mask_variants"] = mask_variants
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline_decode(c5_np, r5_np, d)
        for idx in build_cfgs:  # the oracle's class build on the same workloads, host cores
            result["class_build"][f"config{idx}"]["cpu_baseline"] = cpu_baseline_build(idx)
        for key in class_build_random:
            idx = int(key[len("config"):])
            class_build_random[key]["cpu_baseline"] = cpu_baseline_build(idx, random_table=True)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
