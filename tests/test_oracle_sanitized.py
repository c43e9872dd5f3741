"""The C checker under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a
small paged problem with ragged pages, empty sequences and table padding runs clean and
matches the regular build."""
import os
import subprocess
import sys
import textwrap

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_ubsan(tmp_path):
    lib = tmp_path / "libmarl_oracle_san.so"
    subprocess.check_call(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-fPIC", "-shared", "-std=c99", "-o", str(lib),
                           os.path.join(ROOT, "oracle", "marl_oracle.c"), "-lm"])
    script = textwrap.dedent(f"""
        import ctypes, sys
        import numpy as np
        sys.path.insert(0, {ROOT!r})
        from oracle import reference as ref
        from tests.helpers import Paged, random_logical, to_bf16_bits
        rng = np.random.default_rng(5)
        lg = random_logical(rng, 2, 2, [17, 0], [5, 0, 33, 16], 4, 2)
        pg = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], 2, rng)
        want = ref.decode_attn(to_bf16_bits(lg["q"]), pg.k_bits, pg.v_bits, pg.ptab, pg.stab, pg.plens, pg.slens, pg.gos, 0.1, 4, 2)
        logits = to_bf16_bits(rng.standard_normal((3, 37)).astype(np.float32)); tok = np.array([0, 36, 5], np.int32)
        want_lp = ref.token_logprobs(logits, tok, 0.7)
        ref._lib = None; ref._LIB = {str(lib)!r}; ref.build = lambda force=False: ref._LIB
        got = ref.decode_attn(to_bf16_bits(lg["q"]), pg.k_bits, pg.v_bits, pg.ptab, pg.stab, pg.plens, pg.slens, pg.gos, 0.1, 4, 2, threads=1)
        got_lp = ref.token_logprobs(logits, tok, 0.7, threads=1)
        assert np.abs(got - want).max() <= 1e-13 and np.abs(got_lp - want_lp).max() <= 1e-13
        print("clean")
    """)
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    env = dict(os.environ, LD_PRELOAD=(os.environ.get("LD_PRELOAD", "") + " " + asan).strip(),
               ASAN_OPTIONS="detect_leaks=0", OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-c", script], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0 and "clean" in r.stdout, r.stdout[-2000:]
