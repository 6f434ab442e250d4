"""Helper of test_gpu_parity.py, run as a child process: one short generation on the small bf16 pair, printed as a
digest of every draft logit, target logit, accept result and token.  The parent runs it twice with different routing
switches in the environment (they are read once per process) and compares the digests."""
import hashlib
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import synth  # noqa: E402
import paper_2504_00030_amd as pk  # noqa: E402


def main(batch: int) -> None:
    pk.load()
    cfg = synth.pair("small-bf16")
    Wt, Wd = synth.make_pair_weights(cfg, 0)
    gpu = lambda W: {k: ([t.cuda() for t in v] if isinstance(v, list) else v.cuda()) for k, v in W.items()}
    Wt, Wd = gpu(Wt), gpu(Wd)
    prompts = synth.make_prompts(batch, 300, cfg.target.vocab, 5)  # several 64- and 128-position chunks
    eng = pk.SpecEngine(cfg.target, Wt, cfg.draft, Wd, batch=batch, max_seq=300 + 6 * 17 + 8, gamma_max=16, temperature=1.0,
                        seed=3, accept_mode=pk.ACCEPT_NATURAL, use_graphs=True)
    eng.prefill(prompts)
    h = hashlib.sha256()
    for gamma in (1, 4, 8, 15, 2, 16):
        eng.draft(gamma if batch == 1 else np.full(batch, gamma, dtype=np.int32))
        eng.verify(gamma)
        h.update(np.ascontiguousarray(eng.debug_logits(0)).tobytes())
        A, y, k = eng.accept()
        h.update(np.ascontiguousarray(eng.debug_logits(1)).tobytes())
        for v in (A, y, k):
            h.update(np.ascontiguousarray(v).tobytes())
    for b in range(batch):
        h.update(np.ascontiguousarray(eng.read_tokens(b)).tobytes())
    eng.close()
    print("DIGEST", h.hexdigest(), flush=True)


if __name__ == "__main__":
    main(int(sys.argv[1]))
