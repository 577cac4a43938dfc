"""Schedule strings (the plan input) for the workload families, in the paper's terms:
a sequence of <assignment, loop order> pairs in execution order (Sec. 4.2), CSF operands
written in level order (Sec. 2.1)."""

# mode-0 TTMc of Sec. 5.3, X stored i>j>k:  contract the innermost CSF mode first
TTMC3 = ("T[i,j,s] = X[i,j,k] * U3[k,s] | i,j,k,s ; "
         "Y[i,r,s] = T[i,j,s] * U2[j,r] | i,j,r,s")

# mode-0 MTTKRP of Sec. 5.2 (r is a batch index), X stored i>j>k
MTTKRP3 = ("T[i,j,r] = X[i,j,k] * C[k,r] | i,j,k,r ; "
           "M[i,r] = T[i,j,r] * B[j,r] | i,j,r")

# order-4 TTMc, X stored i>j>k>l; intermediates reduce to order 1 and order 2
TTMC4 = ("T1[i,j,k,t] = X[i,j,k,l] * U3[l,t] | i,j,k,l,t ; "
         "T2[i,j,s,t] = T1[i,j,k,t] * U2[k,s] | i,j,k,s,t ; "
         "Y[i,r,s,t] = T2[i,j,s,t] * U1[j,r] | i,j,r,s,t")

# three-tensor network of Sec. 1 as the tree (U.V).W; U stored i>k>j, W stored k>l>m
SPTN3 = ("T[i,k,l] = U[i,k,j] * V[j,l] | i,k,j,l ; "
         "Z[i,m] = T[i,k,l] * W[k,l,m] | i,k,l,m")


# ---- any output mode by re-rooting the CSF (Sec. 5.2-5.3: one contraction per mode) ------------
#
# The layout is chosen per output mode (Sec. 2.1: the CSF level order fixes the loop order), so
# the output mode goes to the CSF root and the same fused kernels apply.  `levels` names the
# tensor modes in CSF level order, e.g. (1, 2, 0) = output mode 1, then mode 2, leaves on mode 0.

_MODE_NAMES = "ijkl"


def mttkrp3_for(levels):
    """(schedule, operand names) of the order-3 MTTKRP whose CSF level order is `levels`.
    Operands after X: the factor of the leaf mode, then the factor of the middle mode."""
    a, b, c = (_MODE_NAMES[m] for m in levels)
    fb, fc = "F%d" % levels[1], "F%d" % levels[2]
    text = ("T[%s,%s,r] = X[%s,%s,%s] * %s[%s,r] | %s,%s,%s,r ; "
            "M[%s,r] = T[%s,%s,r] * %s[%s,r] | %s,%s,r") % (
        a, b, a, b, c, fc, c, a, b, c, a, a, b, fb, b, a, b)
    return text, ("X", fc, fb)


def ttmc3_for(levels):
    """(schedule, operand names) of the order-3 TTMc whose CSF level order is `levels`; the
    output is [root, rank of the middle mode, rank of the leaf mode]."""
    a, b, c = (_MODE_NAMES[m] for m in levels)
    fb, fc = "F%d" % levels[1], "F%d" % levels[2]
    text = ("T[%s,%s,s] = X[%s,%s,%s] * %s[%s,s] | %s,%s,%s,s ; "
            "Y[%s,r,s] = T[%s,%s,s] * %s[%s,r] | %s,%s,r,s") % (
        a, b, a, b, c, fc, c, a, b, c, a, a, b, fb, b, a, b)
    return text, ("X", fc, fb)


# Sec. 5.1: the three-index integral transformation, every operand sparse, sparse result.
# I stored K > u > v, C stored i > u, P stored m > v, L stored K > i.
SPCHAIN3 = "T[K,i,v] = I[K,u,v] * C[i,u] | K,i,u,v ; E[K,i,m] = T[K,i,v] * P[m,v] | K,i,m,v"
SPCHAIN3_RESTRICTED = ("T[K,i,v] = I[K,u,v] * C[i,u] | K,i,u,v ; F[K,i,v] = T[K,i,v] * L[K,i] | K,i,v ; "
                       "E[K,i,m] = F[K,i,v] * P[m,v] | K,i,m,v")

# Sec. 5.1: the four-index integrals V = E x E over the fitting index K; E stored i > K > m, bound twice
# (two names for one handle), sparse result with levels i > j > m > n.
SPPAIR4 = "V[i,j,m,n] = Ea[i,K,m] * Eb[j,K,n] | i,j,K,m,n"
