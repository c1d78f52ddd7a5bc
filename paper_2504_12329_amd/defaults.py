"""Control parameters of Speculative Thinking as the paper sets them (Appendix C, Appendix D, Section 4.2)."""
N1 = 20                      # tokens the target writes on an Affirmation/Reflection takeover
N2 = 125                     # ... on a Verification takeover
N3 = 125                     # ... on an Excessive-reflection takeover
REFLECTION_THRESHOLD = 15    # negativity counter limit
INITIAL_TARGET_TOKENS = 100  # non-reasoning speculator variant: the target writes the first tokens
