"""CPU oracle (test infrastructure only): see cmoe_oracle.py.  Nothing in the product
package imports this; only tests, the smoke check and the bench's cpu_baseline leg do."""
