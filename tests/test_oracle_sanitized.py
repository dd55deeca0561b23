"""The CPU checker once more under AddressSanitizer and UndefinedBehaviorSanitizer: a small C driver built
with -fsanitize=address,undefined runs the whole pipeline (with and without replacement, int32 and int64
offsets, gather, mean) on a generated graph; any out-of-bounds access, leak or undefined operation fails it."""
import os
import subprocess

import numpy as np
import pytest

from paper_2605_29346_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r'''
#include <stdio.h>
#include <stdlib.h>
#include "zg_oracle.h"
static void *slurp(const char *path, size_t *n) {
    FILE *f = fopen(path, "rb"); if (!f) exit(2);
    fseek(f, 0, SEEK_END); *n = (size_t)ftell(f); fseek(f, 0, SEEK_SET);
    void *p = malloc(*n ? *n : 1); if (fread(p, 1, *n, f) != *n) exit(2); fclose(f); return p;
}
int main(int argc, char **argv) {
    size_t no, ni, ns;
    int is64 = atoi(argv[4]);
    void *off = slurp(argv[1], &no); int32_t *idx = slurp(argv[2], &ni); int32_t *seeds = slurp(argv[3], &ns);
    zgo_graph g = { (int64_t)(no / (is64 ? 8 : 4)) - 1, (int64_t)(ni / 4), off, is64, idx };
    int32_t fan[3] = {4, 3, 2};
    long check = 0;
    for (int rep = 0; rep < 2; ++rep) {
        zgo_blocks b;
        if (zgo_sample_blocks(&g, seeds, (int32_t)(ns / 4), fan, 3, 77, rep, &b)) return 3;
        int dim = 5;
        float *feat = malloc(sizeof(float) * (size_t)g.num_nodes * dim);
        for (int64_t i = 0; i < g.num_nodes * dim; ++i) feat[i] = (float)(i % 17) - 8.0f;
        float *X = malloc(sizeof(float) * (size_t)b.n[3] * dim);
        float *agg = malloc(sizeof(float) * (size_t)b.n[2] * dim);
        zgo_gather(feat, dim, dim, b.S, b.n[3], X, dim);
        zgo_aggregate_mean(b.row_ptr[2], b.col[2], b.n[2], X, dim, dim, agg, dim);
        check += b.n[3] + b.E[0] + b.E[1] + b.E[2] + (long)agg[0];
        free(feat); free(X); free(agg);
        zgo_blocks_free(&b);
    }
    int32_t bad[2] = {1, 1};
    zgo_blocks b;
    if (zgo_sample_blocks(&g, bad, 2, fan, 3, 1, 0, &b) != -1) return 4;   /* duplicate seeds are rejected, nothing leaks */
    printf("ok %ld\n", check);
    free(off); free(idx); free(seeds);
    return 0;
}
'''


@pytest.mark.parametrize("is64", [0, 1])
def test_oracle_under_asan_and_ubsan(tmp_path, is64):
    import torch
    g = W.rmat_graph(3000, 40_000, 9, offsets_dtype=torch.int64 if is64 else torch.int32)
    g.offsets.numpy().tofile(tmp_path / "off.bin")
    g.indices.numpy().tofile(tmp_path / "idx.bin")
    np.random.RandomState(1).permutation(3000)[:50].astype(np.int32).tofile(tmp_path / "seeds.bin")
    (tmp_path / "driver.c").write_text(DRIVER)
    exe = tmp_path / "driver"
    subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
                    "-I", os.path.join(ROOT, "oracle"), str(tmp_path / "driver.c"), os.path.join(ROOT, "oracle", "zg_oracle.c"),
                    "-o", str(exe)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    r = subprocess.run([str(exe), str(tmp_path / "off.bin"), str(tmp_path / "idx.bin"), str(tmp_path / "seeds.bin"), str(is64)],
                       capture_output=True, text=True, env=env)
    assert r.returncode == 0 and r.stdout.startswith("ok"), r.stdout + r.stderr
