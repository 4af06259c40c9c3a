"""Writes listing_address_map_2x3x4.txt: the address map of the paper's parallel-code listing (Section 3.5).

The listing for the permutation (i3,i2,i1) of a 3-index tensor reads A[i1 + i2*lda1 + i3*lda2] and writes
B[i1*ldb2 + i2*ldb1 + i3], with lda1 = size(i1), lda2 = size(i1)*size(i2), ldb1 = size(i3),
ldb2 = size(i3)*size(i2).  This script evaluates exactly that formula for sizes 2 x 3 x 4 and nothing else:
it calls neither the oracle nor the library.  One line per element: offset in A, offset in B.
"""
import os

s1, s2, s3 = 2, 3, 4
lda1, lda2 = s1, s1 * s2
ldb1, ldb2 = s3, s3 * s2
lines = ["# sizes 2 3 4, permutation (i3,i2,i1) = perm (2,1,0); columns: offset in A, offset in B (paper Section 3.5 listing)"]
for i3 in range(s3):
    for i2 in range(s2):
        for i1 in range(s1):
            lines.append(f"{i1 + i2 * lda1 + i3 * lda2} {i1 * ldb2 + i2 * ldb1 + i3}")
with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "listing_address_map_2x3x4.txt"), "w") as f:
    f.write("\n".join(lines) + "\n")
